// Token timelines with the buffer-based, cost-triggered hand-off (Sec. 4.3) in
// class mode: the statistics pass for the (request, column) pairs whose
// source is the column's constrained endpoint in a column with that hand-off.
// The streaming kernels leave these pairs out; the kernel here adds them into
// the same device-wide totals, so a table may mix hand-off kinds freely.  One
// wave walks one request and kind with the general walker (a scan per chunk;
// the hand-off condition compares the delivery slack of every token with the
// migration time).  The pass also leaves 32 bytes per request (BufSummary): a
// hand-off timeline whose running maximum never left 0 delivers at
// round(t tau) like a pure-pacing one, so the histogram passes of the TBT
// selection only walk the others (its walk list names them).  The kernel
// returns at once when the staged table has no such column.
#include <string.h>

#include "disco_tl_general.h"
#include "disco_tl_walk.h"

namespace {

constexpr int TB_BLOCK = 256;                // statistics kernel: 4 waves

struct BufStatsArgs {
    float tau, kt;
    int P;
    int32_t* mig_idx; int32_t* n_src_tok; float* t_last; int32_t* delay_num;
    MigPartial* totals;            // DISCO_NCOPY x 64 device-wide totals, shared with the streaming kernel; nullptr: summaries only
    BufSummary* bufsum;            // per request, written for the requests with a hand-off timeline
    BufCostArgs bc;
    const unsigned* buffer_flag;
};

__global__ __launch_bounds__(TB_BLOCK) void k_tl_stats_buf(TraceView tr, i64 n_tok, int align, const disco_policy* __restrict__ pol,
                                                           BufStatsArgs a)
{
    __shared__ disco_policy spol[DISCO_MAX_COLS];
    __shared__ u64 sh[7 * TB_BLOCK];
    if (*a.buffer_flag == 0u) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int P = a.P;
    if ((int)threadIdx.x < P) spol[threadIdx.x] = pol[threadIdx.x];
    __syncthreads();
    // lane = column
    u64 acc_s_dec = 0, acc_d_dec = 0, acc_repre = 0, acc_srepre = 0, acc_delay = 0, acc_mig = 0;
    double acc_tlast = 0.0;
    const i64 nwaves = (i64)gridDim.x * (TB_BLOCK / 64);
    const i64 nbatch = (tr.n_req + TF_RB - 1) / TF_RB;
    for (i64 bt = (i64)blockIdx.x * (TB_BLOCK / 64) + wave; bt < nbatch; bt += nwaves) {
        const Batch b = load_batch(tr, spol, P, bt * TF_RB, lane);
        u64 walkers = __ballot((b.m[TL_SRV_BUF] | b.m[TL_DEV_BUF]) != 0ull);
        // the first chunk of the next request to walk is loaded while this one is walked
        float ahead[4] = {0.f, 0.f, 0.f, 0.f};
        if (walkers && tr.arr) {
            const int r0 = __ffsll((long long)walkers) - 1;
            first_chunk_load(tr.arr, (i64)bcast_u64((u64)b.off, r0), n_tok, align, bcast_i(b.n, r0), lane, ahead);
        }
        while (walkers) {
            const int rq = __ffsll((long long)walkers) - 1;
            walkers &= walkers - 1;
            const i64 i = bt * TF_RB + rq;
            const int n = bcast_i(b.n, rq), l = bcast_i(b.l, rq);
            const float k = bcast_f(b.k, rq), gd = bcast_f(b.gd, rq), gap = bcast_f(b.gap, rq), s_ttft = bcast_f(b.s, rq);
            const i64 off = tr.arr ? (i64)bcast_u64((u64)b.off, rq) : 0;
            const float chunk[4] = {ahead[0], ahead[1], ahead[2], ahead[3]};
            if (walkers && tr.arr) {
                const int r1 = __ffsll((long long)walkers) - 1;
                first_chunk_load(tr.arr, (i64)bcast_u64((u64)b.off, r1), n_tok, align, bcast_i(b.n, r1), lane, ahead);
            }
            BufSummary bs{0.0f, -1, 0, 0, 0.0f, -1, 0, 0};
#pragma unroll 1
            for (int variant = TL_DEV_BUF; variant >= TL_SRV_BUF; --variant) {
                const u64 mask = bcast_u64(variant == TL_DEV_BUF ? b.m[TL_DEV_BUF] : b.m[TL_SRV_BUF], rq);
                if (!mask) continue;
                auto sink = [](const unsigned*, const bool*) {};
                const TimelineResult res = run_timeline(variant, n, tr.arr, off, n_tok, align, gap, gd, l, k, tr.c, s_ttft, a.bc,
                                                        a.tau, a.kt, lane, nullptr, sink, true, tr.arr ? chunk : nullptr);
                if (variant == TL_DEV_BUF) { bs.M_d = res.M; bs.m_d = buf_m_enc(res.m, res.r0); bs.delay_d = res.delay; }
                else { bs.M_s = res.M; bs.m_s = buf_m_enc(res.m, res.r0); bs.delay_s = res.delay; }
                if (a.totals != nullptr && ((mask >> lane) & 1ull)) {
                    const bool src_dev = variant == TL_DEV_BUF;
                    const bool mig = res.m >= 0;
                    const int nsrc = mig ? res.m + 1 : n;              // tokens produced by the source
                    if (src_dev) { acc_d_dec += (u64)nsrc; acc_s_dec += (u64)(n - nsrc); }
                    else { acc_s_dec += (u64)nsrc; acc_d_dec += (u64)(n - nsrc); }
                    if (mig) {
                        acc_mig += 1;
                        if (src_dev) acc_srepre += (u64)l + (u64)nsrc; else acc_repre += (u64)l + (u64)nsrc;
                        acc_delay += (u64)res.delay;
                    }
                    acc_tlast += (double)res.t_last;
                    if (a.mig_idx) a.mig_idx[(size_t)lane * tr.n_req + i] = mig ? nsrc : -1;
                    if (a.n_src_tok) a.n_src_tok[(size_t)lane * tr.n_req + i] = nsrc;
                    if (a.t_last) a.t_last[(size_t)lane * tr.n_req + i] = res.t_last;
                    if (a.delay_num) a.delay_num[(size_t)lane * tr.n_req + i] = mig ? res.delay : 0;
                }
            }
            if (lane == 0) a.bufsum[i] = bs;                 // (every field is the same on all lanes)
        }
    }
    if (a.totals == nullptr) return;
    // fold the waves of the workgroup, then add into this workgroup's copy of the totals
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
}


}  // namespace

void disco_launch_tl_stats_buf(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a,
                               MigPartial* totals, hipStream_t stream)
{
    BufStatsArgs s;
    memset(&s, 0, sizeof(s));
    s.tau = a.tau; s.kt = a.kt; s.P = a.P;
    s.mig_idx = a.mig_idx; s.n_src_tok = a.n_src_tok; s.t_last = a.t_last; s.delay_num = a.delay_num;
    s.totals = totals;
    s.bufsum = (BufSummary*)a.bufsum;
    s.bc = a.bc;
    s.buffer_flag = a.buffer_flag;
    const i64 per_block = (i64)(TB_BLOCK / 64) * TF_RB;
    i64 b = (v.n_req + per_block - 1) / per_block;
    if (b < 1) b = 1;
    if (b > 2048) b = 2048;
    const int align = (int)(((uintptr_t)v.arr >> 2) & 3);
    hipLaunchKernelGGL(k_tl_stats_buf, dim3((unsigned)b), dim3(TB_BLOCK), 0, stream, v, n_tok, align, pol, s);
}
