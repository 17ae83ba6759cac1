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

constexpr int TS_BLOCK = 256;                // statistics kernel: 4 waves, no histogram
constexpr int TH_BLOCK = 1024;               // histogram kernel: 16 waves share 64 KB of bins

struct WalkOut { int m; float M; };          // hand-off index (-1 none), running maximum over all tokens

// Four arrival offsets of a lane from the token array; `safe` (wave-uniform)
// says that every 16-byte load of the request's window lies inside the array.
__device__ __forceinline__ void load4s(const float* __restrict__ arr, i64 g, i64 n_tok, bool safe, float r[4])
{
    if (safe) {
        const float4 v = *reinterpret_cast<const float4*>(arr + g);
        r[0] = v.x; r[1] = v.y; r[2] = v.z; r[3] = v.w;
    } else {
        load4(arr, g, n_tok, r);
    }
}

// Can the lag trigger be screened by its necessary condition (see walk_hist)?
__device__ __forceinline__ bool lag_fast_ok(int n, float tau, float kt)
{
    return (float)n + 2.0f <= 262144.0f * (kt / tau) && kt >= tau * 0.0009765625f;
}

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

// ------------------------------------------------------------ statistics ---

struct StatsArgs {
    float tau, kt;
    int P;
    int rb;                        // requests per wave batch
    int32_t* mig_idx; int32_t* n_src_tok; float* t_last;
    int32_t* delay_num;            // all zero here: only buffer hand-offs count delayed tokens
    MigPartial* totals;            // DISCO_NCOPY x 64 device-wide totals
};

// Statistics walk of one request and source: the hand-off index and the
// running maximum over all tokens (the last delivery is fma(n-1, tau, M)).
// Only a maximum is needed, not a scan: every lane keeps the maximum of its
// own tokens and the wave reduces once at the end.  The lag trigger is
// evaluated exactly only in chunks that pass the necessary condition stated
// above walk_hist, here with C = u_0 (the first token's shifted arrival, a lower
// bound of every later running maximum).
//   src: 0 token array, 1 constant gap
__device__ __forceinline__ WalkOut walk_stats(bool mem, int n, const float* __restrict__ arr, i64 off, i64 n_tok, int align,
                                              const float first[4], bool have_first, float gap, bool lag, float g_dev,
                                              int l, float k, float c, float tau, float kt, int lane)
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
    float Mlane = ninf;            // maximum of u over this lane's tokens so far
    float C = 0.0f;                // u_0
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
        float i3 = fmaxf(fmaxf(u[0], u[1]), fmaxf(u[2], u[3]));
        if (lag && m < 0) {
            if (e0 == 0) {                                  // u_0 = r_0: element `mis` of lane 0
                const float r0 = mis == 0 ? r[0] : (mis == 1 ? r[1] : (mis == 2 ? r[2] : r[3]));
                C = bcast_f(r0, 0);
            }
            const bool cheap = fast_ok && fabsf(C) <= 262144.0f * kt;
            if (!cheap || __ballot(i3 > C + 0.5f * kt) != 0ull) {
                // exact evaluation: running maximum before each token, then slot and lag as defined (Sec. 4.3 pacing)
                const float before = wave_max_f32(Mlane);
                const float i0 = u[0], i1 = fmaxf(i0, u[1]), i2 = fmaxf(i1, u[2]);
                const float incl = wave_incl_max_dpp(i3, lane);
                const float E = fmaxf(wave_prev(incl, ninf), before);
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
                    i3 = fmaxf(fmaxf(u[0], u[1]), fmaxf(u[2], u[3]));
                }
            }
        }
        Mlane = fmaxf(Mlane, i3);
    }
    return WalkOut{m, wave_max_f32(Mlane)};
}

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
    // (pairs with a buffer hand-off are left to k_tl_stats_buf: acc_n counts the tokens of the pairs handled here)
    u64 acc_s_dec = 0, acc_repre = 0, acc_n = 0, tot_cnt = 0;
    unsigned acc_mig = 0;
    double acc_tlast = 0.0;
    const float tau = a.tau, kt = a.kt;
    const bool mem = tr.arr != nullptr;
    const bool mat = a.mig_idx != nullptr || a.n_src_tok != nullptr || a.t_last != nullptr || a.delay_num != nullptr;
    const i64 nwaves = (i64)gridDim.x * (TS_BLOCK / 64);
    const int rb = a.rb;
    const i64 nbatch = (tr.n_req + rb - 1) / rb;
    for (i64 bt = (i64)blockIdx.x * (TS_BLOCK / 64) + wave; bt < nbatch; bt += nwaves) {
        const Batch b = load_batch(tr, spol, P, bt * rb, lane, rb);
        const int cnt = (int)((tr.n_req - bt * rb < rb) ? (tr.n_req - bt * rb) : rb);
        const u64 srvw = __ballot((b.m[1] | b.m[2]) != 0ull);                  // requests with a server-sourced column
        const u64 memw = mem ? srvw : 0ull;                                    // ... that read the token array
        const bool any_plain = __ballot(b.m[1] != 0ull) != 0ull;
        float pre[4] = {0.f, 0.f, 0.f, 0.f};
        if (memw & 1ull) load_first(tr.arr, (i64)bcast_u64((u64)b.off, 0), bcast_i(b.n, 0), n_tok, align, lane, pre);
#pragma unroll 1
        for (int rq = 0; rq < cnt; ++rq) {
            const i64 i = bt * rb + rq;
            const int n = bcast_i(b.n, rq);
            const float cur[4] = {pre[0], pre[1], pre[2], pre[3]};
            if ((memw >> (rq + 1)) & 1ull)          // the next request's first chunk is loaded while this one is walked
                load_first(tr.arr, (i64)bcast_u64((u64)b.off, rq + 1), bcast_i(b.n, rq + 1), n_tok, align, lane, pre);
            tot_cnt += (u64)(n - 1);
            const u64 mask_lag = bcast_u64(b.m[2], rq);
            const u64 mask_plain = any_plain ? bcast_u64(b.m[1], rq) : 0ull;
            // server source: one walk (with the lag trigger if a column wants it); a second, plain one only if
            // columns without hand-off share the request with a hand-off that fired
            WalkOut lagw{-1, 0.0f}, plainw{-1, 0.0f};
            if ((srvw >> rq) & 1ull) {
                const float gap = mem ? 0.0f : bcast_f(b.gap, rq);
                const bool closed = !mem && pure_pacing(true, gap, tau);        // M = 0, no hand-off
                if (!closed) {
                    const i64 off = mem ? (i64)bcast_u64((u64)b.off, rq) : 0;
                    const bool lag = mask_lag != 0ull;
                    const float gd = bcast_f(b.gd, rq), k = bcast_f(b.k, rq);
                    const int l = bcast_i(b.l, rq);
                    lagw = walk_stats(mem, n, tr.arr, off, n_tok, align, cur, mem, gap, lag, gd, l, k, tr.c, tau, kt, lane);
                    plainw = lagw;
                    if (lag && lagw.m >= 0 && mask_plain != 0ull)
                        plainw = walk_stats(mem, n, tr.arr, off, n_tok, align, cur, false, gap, false, gd, l, k, tr.c, tau, kt, lane);
                }
            }
            // device source: constant gap
            WalkOut devw{-1, 0.0f};
            const u64 mask_dev = bcast_u64(b.m[0], rq);
            if (mask_dev != 0ull) {
                const float gd = bcast_f(b.gd, rq);
                if (!pure_pacing(true, gd, tau))
                    devw = walk_stats(false, n, nullptr, 0, 0, 0, cur, false, gd, false, gd, 0, 0.0f, 0.0f, tau, kt, lane);
            }
            // lane = column picks the timeline of its source
            const bool in_lag = (mask_lag >> lane) & 1ull, in_plain = (mask_plain >> lane) & 1ull;
            const bool in_dev = (mask_dev >> lane) & 1ull;
            if (in_lag || in_plain || in_dev) {
                const WalkOut w = in_lag ? lagw : (in_plain ? plainw : devw);
                const float t_last = __fmaf_rn((float)(n - 1), tau, w.M);
                const int nsrc = in_dev ? 0 : ((w.m >= 0) ? w.m : n);
                acc_s_dec += (u64)nsrc;
                acc_n += (u64)n;
                if (w.m >= 0) { acc_mig += 1u; acc_repre += (u64)bcast_i(b.l, rq) + (u64)w.m; }
                acc_tlast += (double)t_last;
                if (mat) {
                    if (a.mig_idx) a.mig_idx[(size_t)lane * tr.n_req + i] = w.m;
                    if (a.n_src_tok) a.n_src_tok[(size_t)lane * tr.n_req + i] = in_dev ? n : nsrc;
                    if (a.t_last) a.t_last[(size_t)lane * tr.n_req + i] = t_last;
                    if (a.delay_num) a.delay_num[(size_t)lane * tr.n_req + i] = 0;
                }
            }
        }
    }
    // lane = column: fold the waves of the workgroup, then add into this workgroup's copy of the totals
    sh[0 * TS_BLOCK + threadIdx.x] = acc_s_dec; sh[1 * TS_BLOCK + threadIdx.x] = acc_n - acc_s_dec;
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
        x.pad[0] += t->pad[0]; x.pad[1] += t->pad[1];          // server re-prefill, delayed tokens (buffer hand-offs)
        *t = MigPartial{0, 0, 0, 0, 0, 0.0, {0, 0}};
    }
    disco_accum* o = &acc[c];
    o->m_s_dec = (i64)x.s_dec; o->m_d_dec = (i64)x.d_dec; o->m_d_repre = (i64)x.d_repre;
    o->n_migrated = (i64)x.migrated; o->tbt_count = (i64)x.tbt_count; o->tlast_sum = x.tlast_sum;
    o->m_s_repre = (i64)x.pad[0]; o->delay_sum = (i64)x.pad[1];
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
        const Batch b = load_batch(tr, spol, P, bt * rb, lane, rb);
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

void disco_launch_tl_stats_fast(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a,
                                MigPartial* totals, hipStream_t stream)
{
    StatsArgs s;
    memset(&s, 0, sizeof(s));
    s.tau = a.tau; s.kt = a.kt; s.P = a.P;
    s.mig_idx = a.mig_idx; s.n_src_tok = a.n_src_tok; s.t_last = a.t_last; s.delay_num = a.delay_num;
    s.totals = totals;
    s.rb = TF_RB;
    const i64 per_block = (i64)(TS_BLOCK / 64) * s.rb;
    i64 b = (v.n_req + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > 2048) b = 2048;                    // eight resident workgroups per CU
    const int align = (int)(((uintptr_t)v.arr >> 2) & 3);
    hipLaunchKernelGGL(k_tl_stats, dim3((unsigned)b), dim3(TS_BLOCK), 0, stream, v, n_tok, align, pol, s);
    disco_launch_tl_stats_buf(v, n_tok, pol, a, totals, stream);        // pairs with a buffer hand-off, if any
    hipLaunchKernelGGL(k_tl_stats_fin, dim3(1), dim3(64), 0, stream, a.P, totals, a.acc);
}

void disco_launch_tl_hist_fast(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a,
                               hipStream_t stream)
{
    HistArgs h;
    memset(&h, 0, sizeof(h));
    h.tau = a.tau; h.kt = a.kt; h.P = a.P; h.pass = a.pass;
    h.S = a.S; h.ghist = a.ghist; h.ppcnt = a.ppcnt;
    h.rb = tl_batch(v.n_req, 512 * (TH_BLOCK / 64));
    const i64 per_block = (i64)(TH_BLOCK / 64) * h.rb;
    i64 b = (v.n_req + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > 512) b = 512;                      // two resident workgroups per CU
    const int align = (int)(((uintptr_t)v.arr >> 2) & 3);
    hipLaunchKernelGGL(k_tl_hist, dim3((unsigned)b), dim3(TH_BLOCK), 0, stream, v, n_tok, align, pol, h);
}
