// Token timelines with the buffer-based, cost-triggered hand-off (Sec. 4.3) in
// class mode: what the (request, column) pairs whose source is the column's
// constrained endpoint in a column with that hand-off need to know of their
// timeline -- 32 bytes per request (BufSummary: hand-off token, final running
// maximum and delayed tokens of the server-sourced and of the device-sourced
// hand-off timeline).  The kernels of the streaming kinds add these pairs
// into the totals and write their per-pair outputs from the summaries, and a
// hand-off timeline whose running maximum never left 0 delivers at
// round(t tau) like a pure-pacing one, so the histogram passes of the TBT
// selection only walk the others.
//
// Most requests are settled with lane = request:
//   - the cost test (saving > overhead) passes for the tokens 0 .. t_max only
//     (buffer_cost_last); where it never does, the timeline is the source's
//     own, whose final maximum the streaming walk has left;
//   - hand-offs come early (the slack grows by tau minus the source's gap
//     per token): every lane steps through the first tokens of its request
//     with the operations of the general walker (probe_handoff); a hand-off
//     to the device whose tail is provably paced, or the end of the tokens
//     that pass the cost test, settles the request.
// The rest is walked one request per wave with the general walker.  With
// totals, the kernel is the last of the statistics pass to add into them: its
// last workgroup turns them into the columns' accumulators (without a buffer
// column the kernel does only that).
#include <string.h>

#include "disco_tl_general.h"
#include "disco_tl_walk.h"

namespace {

constexpr int TB_BLOCK = 256;                // 4 waves
constexpr int TB_RB = 64;                    // requests per wave batch
constexpr int PROBE_TOKENS = 128;            // tokens a lane steps through before the request is left to a whole wave

struct BufStatsArgs {
    float tau, kt;
    int P, G;                      // columns, columns rounded up to a power of two
    MigPartial* totals;            // DISCO_NCOPY x 64 device-wide totals, shared with the streaming kernels; nullptr: summaries only
    disco_accum* acc;              // with totals: where the workgroup that finishes last puts the columns' totals
    unsigned* ticket;
    BufSummary* bufsum;            // per request, written for the requests with a hand-off timeline
    const TlSummary* summary;      // what the streaming walk found: the source's own timelines
    BufCostArgs bc;
    const unsigned* buffer_flag;
};

// One request of a wave's batch, staged in LDS for the column lanes: its hand-off timelines and the columns that
// use them.
struct BufStaged { u64 cols_s, cols_d; int l, n; int m_s, m_d; int delay_s, delay_d; float M_s, M_d; };

// state 0: nothing settled (the request is walked), 1: no hand-off, 2: hand-off at m with a paced tail
struct ProbeOut { int state; int m; float M; float r0; };

typedef float Float4A __attribute__((ext_vector_type(4), aligned(4)));

// Lane = request: the hand-off test of the general walker on the tokens 0 .. min(limit, PROBE_TOKENS - 1), one
// IEEE operation at a time in the walker's order (u_t, running maximum, delivery, slack, migration time, cost
// test).  limit >= 0: the last token the cost test lets hand off (at most n - 2).
__device__ __forceinline__ ProbeOut probe_handoff(bool active, bool src_dev, int n, const float* __restrict__ arr, i64 off,
                                                  i64 n_tok, float gap_srv, float g_dev, int l, float k, float c, float s_ttft,
                                                  double dc, double cp, float tau, int limit)
{
    const bool from_mem = !src_dev && arr != nullptr;
    const int tend = limit < PROBE_TOKENS - 1 ? limit : PROBE_TOKENS - 1;
    const float gap = src_dev ? g_dev : gap_srv;
    float M = -INFINITY, r_first = 0.0f, M_m = 0.0f, r_m = 0.0f, tm_m = 0.0f;
    int m = -1;
#pragma unroll 1
    for (int t0 = 0; __ballot(active && m < 0 && t0 <= tend) != 0ull; t0 += 4) {
        const bool go = active && m < 0 && t0 <= tend;
        float a4[4] = {0.0f, 0.0f, 0.0f, 0.0f};
        if (go && from_mem) {
            const i64 g = off + t0;
            if (g + 3 < n_tok) {
                const Float4A v = *reinterpret_cast<const Float4A*>(arr + g);
                a4[0] = v.x; a4[1] = v.y; a4[2] = v.z; a4[3] = v.w;
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) a4[q] = g + q < n_tok ? arr[g + q] : 0.0f;
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const int t = t0 + q;
            if (go && m < 0 && t <= tend) {
                const float tf = (float)t;
                const float r = from_mem ? a4[q] : tf * gap;
                const float u = __fmaf_rn(-tf, tau, r);
                M = fmaxf(M, u);
                const float d = __fmaf_rn(tf, tau, M);
                const float slack = d - r;
                const float tm = src_dev ? s_ttft : __fmaf_rn((float)(l + t + 1), k, c);
                if (t == 0) r_first = r;
                if (slack >= tm && buffer_cost_ok(dc, cp, n, l, t)) { m = t; M_m = M; r_m = r; tm_m = tm; }
            }
        }
    }
    ProbeOut o{0, -1, 0.0f, r_first};
    if (!active) return o;
    if (m >= 0) {
        if (!src_dev && paced_tail_proven(r_m, r_first, tm_m, g_dev, tau, (float)m, M_m)) { o.state = 2; o.m = m; o.M = M_m; }
    } else if (tend == limit) {
        o.state = 1;
    }
    return o;
}

__global__ __launch_bounds__(TB_BLOCK) void k_tl_stats_buf(TraceView tr, i64 n_tok, int align, const disco_policy* __restrict__ pol,
                                                           BufStatsArgs a)
{
    __shared__ disco_policy spol[DISCO_MAX_COLS];
    __shared__ __align__(16) BufStaged stage[TB_BLOCK];
    __shared__ u64 sh[7 * TB_BLOCK];
    const int P = a.P;
    if (*a.buffer_flag == 0u) {                              // no such column: the totals are complete as they are
        if (a.totals != nullptr && blockIdx.x == 0) tl_stats_fin(P, a.totals, a.acc);
        return;
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if ((int)threadIdx.x < P) spol[threadIdx.x] = pol[threadIdx.x];
    __syncthreads();
    // totals: lane = sub * G + column, every column lane reads the G requests of its sub-group from LDS
    const int G = a.G, col = lane & (G - 1), sub = lane / G;
    BufStaged* st = stage + wave * 64;
    u64 acc_s_dec = 0, acc_d_dec = 0, acc_repre = 0, acc_srepre = 0, acc_delay = 0, acc_mig = 0;
    double acc_tlast = 0.0;
    const i64 nwaves = (i64)gridDim.x * (TB_BLOCK / 64);
    const i64 nbatch = (tr.n_req + TB_RB - 1) / TB_RB;
    for (i64 bt = (i64)blockIdx.x * (TB_BLOCK / 64) + wave; bt < nbatch; bt += nwaves) {
        const Batch b = load_batch(tr, spol, P, bt * TB_RB, lane, TB_RB, a.summary);
        const bool has_s = b.m[TL_SRV_BUF] != 0ull, has_d = b.m[TL_DEV_BUF] != 0ull;
        if (__ballot(has_s || has_d) == 0ull) continue;
        // lane = request.  Without a hand-off the timeline is the source's own.
        const int lim_s = has_s ? buffer_cost_last(a.bc.dc_srv, a.bc.cp_srv, b.n, b.l) : -1;
        const int lim_d = has_d ? buffer_cost_last(a.bc.dc_dev, a.bc.cp_dev, b.n, b.l) : -1;
        const float r0_dev = 0.0f * b.gd;
        int m_s = -1, m_d = -1, delay_s = 0, delay_d = 0;
        float M_s = has_s ? b.sum.M_plain : 0.0f, M_d = has_d ? b.sum.M_dev : 0.0f;
        bool nz_s = has_s && summary_r0_nonzero(b.sum.m_enc), nz_d = has_d && r0_dev != 0.0f;
        const ProbeOut ps = probe_handoff(lim_s >= 0, false, b.n, tr.arr, b.off, n_tok, b.gap, b.gd, b.l, b.k, tr.c, b.s,
                                          a.bc.dc_srv, a.bc.cp_srv, a.tau, lim_s);
        const ProbeOut pd = probe_handoff(lim_d >= 0, true, b.n, tr.arr, b.off, n_tok, b.gap, b.gd, b.l, b.k, tr.c, b.s,
                                          a.bc.dc_dev, a.bc.cp_dev, a.tau, lim_d);
        if (ps.state == 2) { m_s = ps.m; M_s = ps.M; nz_s = ps.r0 != 0.0f; }
        const bool walk_s = lim_s >= 0 && ps.state == 0, walk_d = lim_d >= 0 && pd.state == 0;
        // one wave per request for the rest; the first chunk of the next one is loaded while this one is walked
        u64 walkers = __ballot(walk_s || walk_d);
        float ahead[4] = {0.f, 0.f, 0.f, 0.f};
        if (walkers && tr.arr) {
            const int r0 = __ffsll((long long)walkers) - 1;
            first_chunk_load(tr.arr, (i64)bcast_u64((u64)b.off, r0), n_tok, align, bcast_i(b.n, r0), lane, ahead);
        }
        while (walkers) {
            const int rq = __ffsll((long long)walkers) - 1;
            walkers &= walkers - 1;
            const int n = bcast_i(b.n, rq), l = bcast_i(b.l, rq);
            const float k = bcast_f(b.k, rq), gd = bcast_f(b.gd, rq), gap = bcast_f(b.gap, rq), s_ttft = bcast_f(b.s, rq);
            const i64 off = tr.arr ? (i64)bcast_u64((u64)b.off, rq) : 0;
            const float chunk[4] = {ahead[0], ahead[1], ahead[2], ahead[3]};
            if (walkers && tr.arr) {
                const int r1 = __ffsll((long long)walkers) - 1;
                first_chunk_load(tr.arr, (i64)bcast_u64((u64)b.off, r1), n_tok, align, bcast_i(b.n, r1), lane, ahead);
            }
            const u64 ws = __ballot(walk_s), wd = __ballot(walk_d);
#pragma unroll 1
            for (int variant = TL_DEV_BUF; variant >= TL_SRV_BUF; --variant) {
                const bool dev = variant == TL_DEV_BUF;
                if ((((dev ? wd : ws) >> rq) & 1ull) == 0ull) continue;
                auto sink = [](const unsigned*, const bool*) {};
                const int limit = bcast_i(dev ? lim_d : lim_s, rq);
                const TimelineResult res = run_timeline(variant, n, tr.arr, off, n_tok, align, gap, gd, l, k, tr.c, s_ttft, a.bc, a.tau,
                                                        a.kt, lane, nullptr, sink, true, tr.arr ? chunk : nullptr, limit);
                if (!res.partial && lane == rq) {             // (partial: no hand-off, the source's own timeline as preset)
                    if (dev) { m_d = res.m; M_d = res.M; delay_d = res.delay; nz_d = res.r0 != 0.0f; }
                    else { m_s = res.m; M_s = res.M; delay_s = res.delay; nz_s = res.r0 != 0.0f; }
                }
            }
        }
        const i64 i = bt * TB_RB + lane;
        if (has_s || has_d)
            a.bufsum[i] = BufSummary{M_s, buf_m_enc(m_s, nz_s ? 1.0f : 0.0f), delay_s, 0, M_d, buf_m_enc(m_d, nz_d ? 1.0f : 0.0f), delay_d, 0};
        if (a.totals == nullptr) continue;
        st[lane] = BufStaged{b.m[TL_SRV_BUF], b.m[TL_DEV_BUF], b.l, b.n, m_s, m_d, delay_s, delay_d, M_s, M_d};
        __builtin_amdgcn_wave_barrier();                     // the staging area is private to the wave
        for (int it = 0; it < G; ++it) {
            const BufStaged r = st[sub * G + it];
#pragma unroll
            for (int dev = 0; dev < 2; ++dev) {
                if ((((dev ? r.cols_d : r.cols_s) >> col) & 1ull) == 0ull) continue;     // (no bit beyond the columns)
                const int m = dev ? r.m_d : r.m_s;
                const int nsrc = m >= 0 ? m + 1 : r.n;       // tokens produced by the source
                if (dev) { acc_d_dec += (u64)nsrc; acc_s_dec += (u64)(r.n - nsrc); }
                else { acc_s_dec += (u64)nsrc; acc_d_dec += (u64)(r.n - nsrc); }
                if (m >= 0) {
                    acc_mig += 1;
                    if (dev) acc_srepre += (u64)r.l + (u64)nsrc; else acc_repre += (u64)r.l + (u64)nsrc;
                    acc_delay += (u64)(dev ? r.delay_d : r.delay_s);
                }
                acc_tlast += (double)__fmaf_rn((float)(r.n - 1), a.tau, dev ? r.M_d : r.M_s);
            }
        }
        __builtin_amdgcn_wave_barrier();
    }
    if (a.totals == nullptr) return;
    // fold the request sub-groups of the wave, the waves of the workgroup, then add into this workgroup's copy of the totals
    for (int mk = G; mk < 64; mk <<= 1) {
        acc_s_dec += shfl_xor_u64(acc_s_dec, mk); acc_d_dec += shfl_xor_u64(acc_d_dec, mk); acc_repre += shfl_xor_u64(acc_repre, mk);
        acc_srepre += shfl_xor_u64(acc_srepre, mk); acc_delay += shfl_xor_u64(acc_delay, mk); acc_mig += shfl_xor_u64(acc_mig, mk);
        acc_tlast += shfl_xor_f64(acc_tlast, mk);
    }
    sh[0 * TB_BLOCK + threadIdx.x] = acc_s_dec; sh[1 * TB_BLOCK + threadIdx.x] = acc_d_dec;
    sh[2 * TB_BLOCK + threadIdx.x] = acc_repre; sh[3 * TB_BLOCK + threadIdx.x] = acc_mig;
    sh[4 * TB_BLOCK + threadIdx.x] = acc_srepre; sh[5 * TB_BLOCK + threadIdx.x] = acc_delay;
    sh[6 * TB_BLOCK + threadIdx.x] = (u64)__double_as_longlong(acc_tlast);
    __syncthreads();
    if ((int)threadIdx.x < P) {
        u64 f[6];
        double tl = 0.0;
        for (int q = 0; q < 6; ++q) f[q] = 0;
        for (int w = 0; w < TB_BLOCK / 64; ++w) {
            for (int q = 0; q < 6; ++q) f[q] += sh[q * TB_BLOCK + w * 64 + threadIdx.x];
            tl += __longlong_as_double((long long)sh[6 * TB_BLOCK + w * 64 + threadIdx.x]);
        }
        MigPartial* t = &a.totals[(blockIdx.x % DISCO_NCOPY) * 64 + threadIdx.x];
        if (f[0]) atomicAdd((unsigned long long*)&t->s_dec, (unsigned long long)f[0]);
        if (f[1]) atomicAdd((unsigned long long*)&t->d_dec, (unsigned long long)f[1]);
        if (f[2]) atomicAdd((unsigned long long*)&t->d_repre, (unsigned long long)f[2]);
        if (f[3]) atomicAdd((unsigned long long*)&t->migrated, (unsigned long long)f[3]);
        if (f[4]) atomicAdd((unsigned long long*)&t->pad[0], (unsigned long long)f[4]);
        if (f[5]) atomicAdd((unsigned long long*)&t->pad[1], (unsigned long long)f[5]);
        if (tl != 0.0) unsafeAtomicAdd(&t->tlast_sum, tl);     // hardware fp64 add; order-dependent in its last bits
    }
    if (!take_last_ticket(a.ticket)) return;
    tl_stats_fin(P, a.totals, a.acc);
    if (threadIdx.x == 0) *a.ticket = 0u;
}

}  // namespace

void disco_launch_tl_stats_buf(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a,
                               MigPartial* totals, hipStream_t stream)
{
    BufStatsArgs s;
    memset(&s, 0, sizeof(s));
    s.tau = a.tau; s.kt = a.kt; s.P = a.P;
    s.G = 1;
    while (s.G < a.P) s.G <<= 1;
    s.totals = totals;
    s.acc = a.acc; s.ticket = a.ticket;
    s.bufsum = (BufSummary*)a.bufsum;
    s.summary = (const TlSummary*)a.summary;
    s.bc = a.bc;
    s.buffer_flag = a.buffer_flag;
    const i64 per_block = (i64)(TB_BLOCK / 64) * TB_RB;
    i64 b = (v.n_req + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > 768) b = 768;                      // what the chip holds at once (3 waves per SIMD): every workgroup ends with a ticket
    const int align = (int)(((uintptr_t)v.arr >> 2) & 3);
    hipLaunchKernelGGL(k_tl_stats_buf, dim3((unsigned)b), dim3(TB_BLOCK), 0, stream, v, n_tok, align, pol, s);
}
