// The general walker of a token timeline (Sec. 4.3): every kind of source and
// hand-off, one scan per chunk, per-token deliveries and gaps handed to a
// sink.  Used by the general kernel and by the kernels that walk the buffer
// hand-off timelines; the lag-trigger and plain timelines of the streaming
// kernels have leaner walkers of their own.
#pragma once
#include "disco_tl_device.h"

namespace {

// ------------------------------------------------------------- timeline ----

// M: final running maximum, r0: arrival of token 0; partial: the walk ended at the caller's token limit without a
// hand-off (m = -1; t_last, delay and M are not set)
struct TimelineResult { int m; float t_last; int delay; float M; float r0; int partial; };

// Prices behind the buffer hand-off's cost test (Sec. 4.3: saving > overhead).
typedef BufCostArgs BufCost;

// The cost test at token t of a request with prompt l and n output tokens: the decode saving on the n - 1 - t
// tokens still to come against the target's prefill of the l + t + 1 tokens so far.
__device__ __forceinline__ bool buffer_cost_ok(double dc, double cp, int n, int l, int t)
{
    const double saved = dc * (double)(n - 1 - t);
    const double overhead = cp * (double)(l + t + 1);
    return saved > overhead;
}

// Last token at which the cost test can pass, -1 if none.  For dc > 0 and cp >= 0 the saving does not grow and the
// overhead does not shrink with t (a product with a constant of fixed sign is monotone under rounding), so the
// tokens that pass are 0 .. t_max: bisection with the test itself.  Other signs: no bound (n - 2, the last
// token a hand-off may follow).
__device__ __forceinline__ int buffer_cost_last(double dc, double cp, int n, int l)
{
    if (n < 2) return -1;
    if (!(dc > 0.0 && cp >= 0.0)) return n - 2;
    if (!buffer_cost_ok(dc, cp, n, l, 0)) return -1;
    int lo = 0, hi = n - 1;                 // passes at lo; hi: fails or is past the last candidate
    while (hi - lo > 1) {
        const int mid = lo + ((hi - lo) >> 1);
        if (buffer_cost_ok(dc, cp, n, l, mid)) lo = mid; else hi = mid;
    }
    return lo;
}

// Paced tail behind a buffer hand-off to the device at token m (see run_timeline): r_m, r_first the arrivals of
// tokens m and 0, tm the migration time, M_m the running maximum through token m.
__device__ __forceinline__ bool paced_tail_proven(float r_m, float r_first, float tm, float g_dev, float tau, float m_f, float M_m)
{
    const float reach = __fmaf_rn(m_f + 2.0f, tau, fabsf(M_m));
    return r_m >= 0.0f && r_first >= 0.0f && tm >= 0.0f && g_dev >= 0.0f && tau - g_dev >= 9.5367431640625e-07f * reach;
}

// Timeline of one request and source.
//   variant 0: device source, 1: server source, 2: server source with the lag trigger,
//           3: server source with the buffer hand-off (target device),
//           4: device source with the buffer hand-off (target server)
//   arr/off/n_tok: CSR token array of the server or arr == nullptr (constant gap `gap_srv`)
//   deliv: nullable, delivery offsets of the request's tokens
//   sink(key[4], ok[4]): called once per chunk by all lanes (ok marks real gaps)
// Returns m = the lag trigger's first device token, or the last source token of a buffer hand-off.
//   stop_paced: the caller needs only the result (no deliveries, no gaps): a hand-off to the device whose tail is
//           provably paced ends the walk (see below)
//   first_chunk: nullable; this lane's four elements of the first chunk, loaded by the caller exactly as
//           first_chunk_load does (so that the load can be in flight while another request is walked)
//   t_limit: a buffer hand-off is known to be impossible after this token (buffer_cost_last): a walk that has
//           tested every token up to it without a hand-off ends with `partial` set, unless it is in its last
//           chunk anyway; for callers that have the final running maximum of the source's own timeline from
//           elsewhere
//
// Paced tail behind a buffer hand-off to the device (variant 3).  At the hand-off token m the slack
// S = fl(delta_m - r_m) covers the migration time TM, the target's arrivals are R_t = fma(t - m, g, fl(r_m + TM))
// and delta_m = fl(m tau + M_m).  With e = 2^-24 and every quantity non-negative (first arrival, r_m, TM, g: checked),
//   fl(r_m + TM) <= (r_m + S)(1 + e) <= delta_m (1 + e)^2 <= (m tau + M_m)(1 + e)^3,
// so for t = m + j:  fl(R_t - t tau) <= M_m - j (tau - g) + 6 e (t tau + M_m), and the pacing slot
// fl(delta_{t-1} + tau) >= t tau + M_m - 2 e (t tau + M_m).  If tau - g >= 2^-20 ((m + 2) tau + M_m), i.e. 16 e
// of the largest magnitude, then j (tau - g) exceeds both error terms for every j >= 1: u_t = fl(R_t - t tau)
// <= M_m (the running maximum stays M_m, the last delivery is fma(n - 1, tau, M_m)) and R_t is never above its
// pacing slot (no delayed token).  Requests that miss the condition are walked to the end.
// This lane's elements of the first chunk of a request's window in the token array (zeros beyond the request).
__device__ __forceinline__ void first_chunk_load(const float* __restrict__ arr, i64 off, i64 n_tok, int align, int n, int lane,
                                                 float out[4])
{
    const int mis = (int)((off + align) & 3);
    out[0] = out[1] = out[2] = out[3] = 0.0f;
    if (4 * lane - mis < n) load4(arr, off - mis + 4 * lane, n_tok, out);
}

template <class Sink>
__device__ __forceinline__ TimelineResult run_timeline(int variant, int n, const float* __restrict__ arr, i64 off, i64 n_tok,
                                                       int align, float gap_srv, float g_dev, int l, float k, float c,
                                                       float s_ttft, const BufCost& bc, float tau, float kt, int lane,
                                                       float* __restrict__ deliv, Sink&& sink, bool stop_paced = false,
                                                       const float* first_chunk = nullptr, int t_limit = 0x7FFFFFFF)
{
    const bool src_dev = variant == 0 || variant == 4;
    const bool buffer = variant >= 3;
    const bool from_mem = !src_dev && arr != nullptr;       // source arrivals come from the token array
    const bool tgt_mem = variant == 4 && arr != nullptr;    // the target's arrivals follow the token array
    const bool use_mem = from_mem || tgt_mem;
    const double dc = variant == 3 ? bc.dc_srv : bc.dc_dev, cp = variant == 3 ? bc.cp_srv : bc.cp_dev;
    // element 0 of the window is the aligned-down start: the first `mis` elements precede the request
    const int mis = use_mem ? (int)((off + align) & 3) : 0;
    const i64 gbase = off - mis + 4 * lane;
    float carryM = -INFINITY, carryD = INFINITY, base = 0.0f, t_last = 0.0f, a_m = 0.0f, r_first = 0.0f;
    int m = -1, delay = 0;
    float nxt[4] = {0.f, 0.f, 0.f, 0.f};
    if (use_mem && first_chunk != nullptr) {
#pragma unroll
        for (int q = 0; q < 4; ++q) nxt[q] = first_chunk[q];
    } else if (use_mem && 4 * lane - mis < n) {
        load4(arr, gbase, n_tok, nxt);
    }
    const int total = n + mis;
    for (int e0 = 0; e0 < total; e0 += 256) {
        const int tb = e0 + 4 * lane - mis;                 // token index of this lane's first element
        float r[4], a[4];
        int tk[4];
        float tf[4];
        bool val[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) { tk[q] = tb + q; tf[q] = (float)tk[q]; val[q] = tk[q] >= 0 && tk[q] < n; a[q] = 0.0f; }
        if (use_mem && (m < 0 || tgt_mem)) {
#pragma unroll
            for (int q = 0; q < 4; ++q) a[q] = nxt[q];
            if (e0 + 256 < total && tb + 256 < n) load4(arr, gbase + e0 + 256, n_tok, nxt);   // next chunk in flight
        }
        // arrivals of the spliced sequence
        auto arrival = [&](int q) -> float {
            if (m >= 0 && !buffer) return __fmaf_rn((float)(tk[q] - m + 1), g_dev, base);      // lag: device from token m
            if (m >= 0 && tk[q] > m) {                                                           // buffer: target after token m
                if (variant == 3) return __fmaf_rn((float)(tk[q] - m), g_dev, base);
                if (tgt_mem) { const float since = a[q] - a_m; return base + since; }
                return __fmaf_rn((float)(tk[q] - m), gap_srv, base);
            }
            if (src_dev) return tf[q] * g_dev;
            return from_mem ? a[q] : tf[q] * gap_srv;
        };
#pragma unroll
        for (int q = 0; q < 4; ++q) r[q] = val[q] ? arrival(q) : -INFINITY;
        if (e0 == 0) {                      // token 0 is element `mis` of lane 0
            const float rf = mis == 0 ? r[0] : (mis == 1 ? r[1] : (mis == 2 ? r[2] : r[3]));
            r_first = bcast_f(rf, 0);
        }
        float d[4], prev[4], Mq[4];
        float Mlast;
        auto scan = [&]() {
            float u[4], mx[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) u[q] = __fmaf_rn(-tf[q], tau, r[q]);      // -inf for lanes outside the request
            mx[0] = u[0]; mx[1] = fmaxf(mx[0], u[1]); mx[2] = fmaxf(mx[1], u[2]); mx[3] = fmaxf(mx[2], u[3]);
            const float incl = wave_incl_max_dpp(mx[3], lane);
            const float excl = fmaxf(wave_prev(incl, -INFINITY), carryM);
#pragma unroll
            for (int q = 0; q < 4; ++q) { Mq[q] = fmaxf(excl, mx[q]); d[q] = __fmaf_rn(tf[q], tau, Mq[q]); }
            Mlast = fmaxf(excl, mx[3]);
            prev[0] = wave_prev(d[3], carryD);
            prev[1] = d[0]; prev[2] = d[1]; prev[3] = d[2];
        };
        scan();
        if (variant == 2 && m < 0) {
            bool trig[4];
            float slot[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                slot[q] = prev[q] + tau;
                const float lag = r[q] - slot[q];
                trig[q] = val[q] && tk[q] >= 1 && lag > kt;
            }
            const u64 any = __ballot(trig[0] || trig[1] || trig[2] || trig[3]);
            if (any) {
                const int ml = __ffsll((long long)any) - 1;
                const int qf = trig[0] ? 0 : (trig[1] ? 1 : (trig[2] ? 2 : 3));
                const float sl = trig[0] ? slot[0] : (trig[1] ? slot[1] : (trig[2] ? slot[2] : slot[3]));
                const int q_m = bcast_i(qf, ml);
                m = bcast_i(tb, ml) + q_m;
                // hand-off: decided once the token is kappa*tau overdue; the device re-prefills the
                // prompt plus the m tokens already produced, then generates at its own pace
                const float t_dec = bcast_f(sl, ml) + kt;
                const float t_mig = __fmaf_rn((float)(l + m), k, c);
                base = t_dec + t_mig;
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (tk[q] >= m) r[q] = val[q] ? arrival(q) : -INFINITY;
                scan();
            }
        }
        if (buffer && m < 0) {
            // buffer hand-off after the first token whose playback time ahead covers the migration time and whose
            // remaining decode saving exceeds the target's prefill overhead
            bool trig[4];
            float tm[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const float slack = d[q] - r[q];
                tm[q] = variant == 4 ? s_ttft : __fmaf_rn((float)(l + tk[q] + 1), k, c);
                trig[q] = val[q] && tk[q] + 1 < n && slack >= tm[q] && buffer_cost_ok(dc, cp, n, l, tk[q]);
            }
            const u64 any = __ballot(trig[0] || trig[1] || trig[2] || trig[3]);
            if (any) {
                const int ml = __ffsll((long long)any) - 1;
                const int qf = trig[0] ? 0 : (trig[1] ? 1 : (trig[2] ? 2 : 3));
                const float rm = trig[0] ? r[0] : (trig[1] ? r[1] : (trig[2] ? r[2] : r[3]));
                const float tmm = trig[0] ? tm[0] : (trig[1] ? tm[1] : (trig[2] ? tm[2] : tm[3]));
                const float am = trig[0] ? a[0] : (trig[1] ? a[1] : (trig[2] ? a[2] : a[3]));
                m = bcast_i(tb, ml) + bcast_i(qf, ml);
                base = bcast_f(rm, ml) + bcast_f(tmm, ml);
                a_m = bcast_f(am, ml);
                if (stop_paced && variant == 3) {
                    const float tfm = trig[0] ? tf[0] : (trig[1] ? tf[1] : (trig[2] ? tf[2] : tf[3]));
                    // M_m: the running maximum through token m, from the hand-off lane
                    const float mq = trig[0] ? Mq[0] : (trig[1] ? Mq[1] : (trig[2] ? Mq[2] : Mq[3]));
                    const float M_m = bcast_f(mq, ml);
                    const float r_m = bcast_f(rm, ml);
                    if (paced_tail_proven(r_m, r_first, bcast_f(tmm, ml), g_dev, tau, bcast_f(tfm, ml), M_m)) {
                        const float tl_ = __fmaf_rn((float)(n - 1), tau, M_m);
                        return TimelineResult{m, tl_, 0, M_m, r_first, 0};
                    }
                }
#pragma unroll
                for (int q = 0; q < 4; ++q)
                    if (tk[q] > m) r[q] = val[q] ? arrival(q) : -INFINITY;
                scan();
            }
        }
        if (buffer && m < 0 && e0 + 255 - mis >= t_limit && e0 + 256 < total)
            return TimelineResult{-1, 0.0f, 0, 0.0f, r_first, 1};
        unsigned key[4];
        bool ok[4];
        bool late[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const float gap = d[q] - prev[q];
            key[q] = f2u(gap);
            ok[q] = val[q] && tk[q] >= 1;
            // delayed (Sec. 5.2, delay_num): the token arrives after its pacing slot -- decided on the arrival, so
            // that the one-ulp scatter of paced gaps around tau cannot count
            const float slot = prev[q] + tau;
            const float lag = r[q] - slot;
            late[q] = buffer && m >= 0 && val[q] && tk[q] > m && lag > 0.0f;
            if (deliv && val[q]) deliv[tk[q]] = d[q];
        }
        if (buffer && m >= 0)
            delay += __popcll(__ballot(late[0])) + __popcll(__ballot(late[1])) + __popcll(__ballot(late[2])) +
                     __popcll(__ballot(late[3]));
        sink(key, ok);
        carryM = bcast_f(Mlast, 63);
        carryD = bcast_f(d[3], 63);
        if (e0 + 256 >= total) {            // last chunk: delivery offset of token n-1
            const int e = n - 1 + mis - e0;
            const int q_l = e & 3;
            const float dl = q_l == 0 ? d[0] : (q_l == 1 ? d[1] : (q_l == 2 ? d[2] : d[3]));
            t_last = bcast_f(dl, e >> 2);
        }
    }
    return TimelineResult{m, t_last, delay, carryM, r_first, 0};
}

// Pure pacing: a source whose constant gap is safely below tau (gap < 0.999 tau).
// Then u_0 = 0 and u_t = round(round(t gap) - t tau) < 0 for t >= 1 (the
// product's rounding error is below 2^-24 relative, far inside the 1e-3
// margin), the running maximum stays 0, delta_t = fma(t, tau, 0) = round(t tau),
// and no token is ever overdue.  The result depends on n alone.
template <class Sink>
__device__ __forceinline__ TimelineResult run_pure_pacing(int n, float tau, int lane, float* __restrict__ deliv, bool need_keys,
                                                          Sink&& sink)
{
    if (need_keys || deliv) {
        for (int e0 = 0; e0 < n; e0 += 256) {
            unsigned key[4];
            bool ok[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const int t = e0 + 4 * lane + q;
                const float dq = (float)t * tau;
                const float pq = (float)(t - 1) * tau;
                key[q] = f2u(dq - pq);
                ok[q] = t >= 1 && t < n;
                if (deliv && t < n) deliv[t] = dq;
            }
            if (need_keys) sink(key, ok);
        }
    }
    return TimelineResult{-1, (float)(n - 1) * tau, 0, 0.0f, 0.0f, 0};
}

}  // namespace
