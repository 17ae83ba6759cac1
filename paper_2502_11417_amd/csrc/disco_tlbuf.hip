// Token timelines with the buffer-based, cost-triggered hand-off (Sec. 4.3) in
// class mode: the statistics pass and the TBT histogram passes for the
// (request, column) pairs whose source is the column's constrained endpoint
// in a column with that hand-off.  The streaming kernels leave these pairs
// out; the kernels here add them into the same device-wide totals and
// histogram rows, so a table may mix hand-off kinds freely.  One wave walks
// one request and kind with the general walker (a scan per chunk; the hand-off
// condition compares the delivery slack of every token with the migration
// time).  The statistics pass also leaves 32 bytes per request (BufSummary):
// a hand-off timeline whose running maximum never left 0 delivers at
// round(t tau) like a pure-pacing one, so the histogram passes only walk the
// others (the walk list of the TBT selection names them).  Both kernels
// return at once when the staged table has no such column.
#include <string.h>

#include "disco_tl_general.h"
#include "disco_tl_walk.h"

namespace {

constexpr int TB_BLOCK = 256;                // statistics kernel: 4 waves
constexpr int TBH_BLOCK = 1024;              // histogram kernel: 16 waves share the LDS bins

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

struct BufHistArgs {
    HistArgs h;
    BufCostArgs bc;
    const unsigned* buffer_flag;
};

// One histogram pass over the hand-off timelines that have tokens to walk: bytes 3 and 4 of a request's
// descriptor name the LDS rows of its two hand-off kinds, the walk list of the selection names the requests.
__global__ __launch_bounds__(TBH_BLOCK) void k_tl_hist_buf(TraceView tr, i64 n_tok, int align, BufHistArgs ba)
{
    __shared__ __align__(16) unsigned smem[DISCO_TL_HIST_WORDS];
    const HistArgs& a = ba.h;
    const TlSel* tl = &a.S->tl;
    const int width = tl->width;
    if (*ba.buffer_flag == 0u || width <= 0 || tl->fallback) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ncls = tl->ncls, nwalk = tl->nwalk;
    HistCtx h;
    h.hist = smem; h.width = width; h.shift = tl->shift; h.up = h.shift + width;
    h.G = tl->G < DISCO_MAX_GRP ? tl->G : DISCO_MAX_GRP;
    h.stride = (unsigned)nwalk << width;
    h.key_lo = tl->key_lo; h.key_cap = tl->window ? (1u << tl->window) : 0xFFFFFFFFu;
    for (int k = 0; k < DISCO_MAX_GRP; ++k) h.grp_prefix[k] = tl->grp_prefix[k];
    const int words = (h.G * nwalk) << width;
    for (int i = threadIdx.x; i < words; i += TBH_BLOCK) smem[i] = 0u;
    __syncthreads();
    const i64 nwaves = (i64)gridDim.x * (TBH_BLOCK / 64);
    const i64 nfront = (i64)tl->nlist, nlist = nfront + (i64)tl->nlist_back;
    i64 rb = (nlist + nwaves - 1) / nwaves;
    rb = rb < 1 ? 1 : (rb > 64 ? 64 : rb);
    const i64 nround = (nlist + rb * nwaves - 1) / (rb * nwaves);
    for (i64 rnd = 0; rnd < nround; ++rnd) {
        const i64 gw = (i64)blockIdx.x * (TBH_BLOCK / 64) + wave;
        const i64 j = rnd * rb * nwaves + gw + (i64)lane * nwaves;
        const bool mine = lane < rb && j < nlist;
        const i64 il = mine ? (i64)walk_list_entry(a.list, tr.n_req, nfront, j) : 0;
        const unsigned desc = mine ? (unsigned)((a.desc[il] >> 24) & 0xFFFFull) : 0xFFFFu;
        u64 walkers = __ballot(desc != 0xFFFFu);
        if (!walkers) continue;
        int l_v = 0, n_v = 1;
        float k_v = tr.k_s, gd_v = tr.g_s, gap_v = 0.0f, s_v = 0.0f;
        i64 off_v = 0;
        if (desc != 0xFFFFu) {
            l_v = tr.l[il]; n_v = tr.n[il]; s_v = tr.s[il];
            if (tr.k) k_v = tr.k[il];
            if (tr.g) gd_v = tr.g[il];
            if (tr.off) off_v = tr.off[il];
            if (tr.tbt) gap_v = tr.tbt[il];
        }
        while (walkers) {
            const int rq = __ffsll((long long)walkers) - 1;
            walkers &= walkers - 1;
            const unsigned dsc = (unsigned)bcast_i((int)desc, rq);
            const int n = bcast_i(n_v, rq), l = bcast_i(l_v, rq);
            const float k = bcast_f(k_v, rq), gd = bcast_f(gd_v, rq), gap = bcast_f(gap_v, rq), s_ttft = bcast_f(s_v, rq);
            const i64 off = tr.arr ? (i64)bcast_u64((u64)off_v, rq) : 0;
#pragma unroll 1
            for (int kind = 1; kind >= 0; --kind) {
                const unsigned sl = (dsc >> (8 * kind)) & 0xFFu;
                if (sl == 0xFFu) continue;
                const unsigned row_base = sl << width;
                auto sink = [&](const unsigned key[4], const bool ok[4]) {
                    const unsigned kk[4] = {ok[0] ? key[0] : KEY_SKIP, ok[1] ? key[1] : KEY_SKIP, ok[2] ? key[2] : KEY_SKIP,
                                            ok[3] ? key[3] : KEY_SKIP};
                    hist_keys(h, kk, row_base, lane);
                };
                (void)run_timeline(TL_SRV_BUF + kind, n, tr.arr, off, n_tok, align, gap, gd, l, k, tr.c, s_ttft, ba.bc, a.tau, a.kt,
                                   lane, nullptr, sink);
            }
        }
    }
    __syncthreads();
    // LDS rows (group, walked class) -> device-wide rows (group, class)
    const unsigned dmask = (1u << width) - 1u;
    for (int i = threadIdx.x; i < words; i += TBH_BLOCK) {
        const unsigned cnt = smem[i];
        if (!cnt) continue;
        const int row = i >> width;
        const int g = row / nwalk, sl = row - g * nwalk;
        const int c = tl->slot_cls[sl];
        atomicAdd(&a.ghist[((size_t)(g * ncls + c) << width) | ((unsigned)i & dmask)], cnt);
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

void disco_launch_tl_hist_buf(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a,
                              hipStream_t stream)
{
    BufHistArgs h;
    memset(&h, 0, sizeof(h));
    h.h.tau = a.tau; h.h.kt = a.kt; h.h.P = a.P; h.h.pass = a.pass;
    h.h.S = a.S; h.h.ghist = a.ghist;
    h.h.desc = a.desc; h.h.list = a.list;
    h.bc = a.bc;
    h.buffer_flag = a.buffer_flag;
    (void)pol;
    i64 b = (v.n_req + TBH_BLOCK / 64 - 1) / (TBH_BLOCK / 64);    // at most one request per wave
    if (b < 1) b = 1;
    const i64 cap = a.pass < 2 ? 512 : 64;                       // (the late passes normally return at once)
    if (b > cap) b = cap;
    const int align = (int)(((uintptr_t)v.arr >> 2) & 3);
    hipLaunchKernelGGL(k_tl_hist_buf, dim3((unsigned)b), dim3(TBH_BLOCK), 0, stream, v, n_tok, align, h);
}
