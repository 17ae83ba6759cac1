// Token timelines (Sec. 4.3), the general workgroup body: everything the
// streaming kernels leave out -- the statistics pass that also writes the
// per-token deliveries of one column, and the TBT histogram passes with one
// histogram per (column, quantile) slot, used when the column sets of the
// table do not fit the class scheme.  Shared by the general kernel and by the
// kernels that run a histogram pass of every kind in one launch.
//
// One wave walks one request at a time in chunks of 256 tokens, four
// consecutive tokens per lane.  The delivery recurrence
// delta_t = max(r_t, delta_{t-1} + tau) is evaluated in the shifted domain
// u_t = r_t - t tau, where it is a running maximum: a 4-element scan in
// registers, a DPP scan across the wave, a carried maximum between chunks.
// `max` is exact and associative, so the result does not depend on the scan
// order and equals the sequential definition bit for bit.  Lane j < P keeps
// column j's totals in registers.
#pragma once
#include "disco_tl_general.h"

namespace {

// ------------------------------------------------------------ histogram ----

// What a histogram pass needs, cached in LDS / registers per workgroup.
struct SlotHistCtx {
    unsigned* hist;          // LDS bins
    int shift, width, up;    // digit of this pass; up = shift + width
    int nq;
    unsigned key_lo, key_cap; // see tbt_key
    const unsigned* sprefix; // LDS, per slot
    const int* slive;        // LDS, per slot
};

// Fallback path: one histogram per (column, quantile) slot; a key counts for a
// slot if its upper bits equal the slot's prefix.  Columns that share a prefix
// are served together; equal bins are counted with ballots, lane = column adds.
__device__ __forceinline__ void hist_keys_cols(const SlotHistCtx& h, const unsigned key[4], const bool ok[4], u64 cols, int lane)
{
    const unsigned dmask = (1u << h.width) - 1u;
    for (int qi = 0; qi < h.nq; ++qi) {
        u64 cm = cols;
        while (cm) {
            const int c0 = __ffsll((long long)cm) - 1;
            const unsigned pf = h.sprefix[c0 * h.nq + qi];
            u64 grp = 0ull;
            for (u64 rest = cm; rest; rest &= rest - 1) {
                const int c1 = __ffsll((long long)rest) - 1;
                if (h.sprefix[c1 * h.nq + qi] == pf && h.slive[c1 * h.nq + qi]) grp |= 1ull << c1;
            }
            cm &= ~(grp | (1ull << c0));
            if (!grp) continue;
            unsigned bin[4];
            bool pend[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const unsigned kk = tbt_key(key[k], h.key_lo, h.key_cap);
                bin[k] = (kk >> h.shift) & dmask;
                pend[k] = ok[k] && (kk >> h.up) == pf;           // clamped keys have a bit above every prefix
            }
            u64 todo = __ballot(pend[0] || pend[1] || pend[2] || pend[3]);
            while (todo) {
                const int leader = __ffsll((long long)todo) - 1;
                const unsigned mine = pend[0] ? bin[0] : (pend[1] ? bin[1] : (pend[2] ? bin[2] : bin[3]));
                const unsigned b0 = (unsigned)bcast_i((int)mine, leader);
                unsigned cnt = 0;
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const bool same = pend[k] && bin[k] == b0;
                    cnt += (unsigned)__popcll(__ballot(same));
                    pend[k] = pend[k] && !same;
                }
                if ((grp >> lane) & 1ull) atomicAdd(&h.hist[(((unsigned)lane * h.nq + qi) << h.width) | b0], cnt);
                todo = __ballot(pend[0] || pend[1] || pend[2] || pend[3]);
            }
        }
    }
}

constexpr int TL_BLOCK = 1024;
constexpr int TL_WAVES = TL_BLOCK / 64;
constexpr int TL_RB = 16;                   // requests per wave batch

// LDS of a workgroup that runs the general body.
struct TimelineLds {
    unsigned sprefix[DISCO_MAX_SLOTS];
    int slive[DISCO_MAX_SLOTS];
    disco_policy spol[DISCO_MAX_COLS];
};

// Workgroup `bid` of `nblk` (the statistics pass, a.pass < 0, takes the last-ticket test over the whole grid:
// it must be called by every workgroup of the launch, bid = blockIdx.x; HIST_ONLY leaves that pass out of the
// code).  `smem`: DISCO_TL_HIST_WORDS words of LDS.
template <bool HIST_ONLY>
__device__ __forceinline__ void timeline_body(unsigned* smem, TimelineLds& lds, const TraceView& tr, i64 n_tok, int align,
                                              const disco_policy* __restrict__ pol, const TimelineArgs& a, unsigned bid,
                                              unsigned nblk)
{
    unsigned* sprefix = lds.sprefix;
    int* slive = lds.slive;
    disco_policy* spol = lds.spol;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int P = a.P, nq = a.nq;
    if ((int)threadIdx.x < P) spol[threadIdx.x] = pol[threadIdx.x];
    const bool hist_pass = HIST_ONLY || a.pass >= 0;       // pass -1: statistics
    SlotHistCtx h;
    h.hist = smem; h.shift = 0; h.width = 0; h.up = 0; h.nq = nq; h.key_lo = 0u; h.key_cap = 0xFFFFFFFFu;
    h.sprefix = sprefix; h.slive = slive;
    if (hist_pass) {
        const TlSel* tl = &a.S->tl;
        h.width = tl->width;
        if (h.width <= 0 || !tl->fallback) return;     // selection finished, or class histograms (other kernel)
        h.shift = tl->shift;
        h.up = h.shift + h.width;
        h.key_lo = tl->key_lo; h.key_cap = tl->window ? (1u << tl->window) : 0xFFFFFFFFu;
        const int words = (P * nq) << h.width;
        for (int i = threadIdx.x; i < words; i += TL_BLOCK) smem[i] = 0u;
        for (int i = threadIdx.x; i < P * nq; i += TL_BLOCK) {
            const SelSlot sl = a.S->slot[1][i];
            sprefix[i] = sl.prefix;
            slive[i] = !sl.done;
        }
    }
    __syncthreads();
    u64 acc_s_dec = 0, acc_d_dec = 0, acc_repre = 0, acc_srepre = 0, acc_delay = 0, acc_mig = 0, acc_cnt = 0;
    double acc_tlast = 0.0;
    const i64 nwaves = (i64)nblk * TL_WAVES;
    // A wave takes TL_RB consecutive requests at a time.  Phase A, lane = request: the fields are
    // loaded coalesced and every column's dispatch is evaluated, giving the three column sets of the
    // request (device source, server source, server source with lag hand-off).  Phase B walks the
    // requests one by one with the whole wave on the tokens.
    const i64 nbatch = (tr.n_req + TL_RB - 1) / TL_RB;
    for (i64 bt = (i64)bid * TL_WAVES + wave; bt < nbatch; bt += nwaves) {
        const i64 ia = bt * TL_RB + lane;
        const bool va = lane < TL_RB && ia < tr.n_req;
        int l_v = 0, n_v = 1;
        float s_v = 0.0f, k_v = tr.k_s, g_v = tr.g_s, gap_v = 0.0f;
        i64 off_v = 0;
        if (va) {
            l_v = tr.l[ia]; n_v = tr.n[ia]; s_v = tr.s[ia];
            if (tr.k) k_v = tr.k[ia];
            if (tr.g) g_v = tr.g[ia];
            if (tr.off) off_v = tr.off[ia];
            if (tr.tbt) gap_v = tr.tbt[ia];
        }
        // column sets by kind of timeline
        u64 m_v[TL_KINDS];
        request_sets(spol, P, l_v, s_v, __fmaf_rn((float)l_v, k_v, tr.c), ia, m_v);
        if (!va) m_v[0] = m_v[1] = m_v[2] = m_v[3] = m_v[4] = 0ull;
        const int cnt = (int)((tr.n_req - bt * TL_RB < TL_RB) ? (tr.n_req - bt * TL_RB) : TL_RB);
#pragma unroll 1
      for (int rq = 0; rq < cnt; ++rq) {
        const i64 i = bt * TL_RB + rq;
        const int l = bcast_i(l_v, rq), n = bcast_i(n_v, rq);
        const float k = bcast_f(k_v, rq), gd = bcast_f(g_v, rq);
        const float gap_src = bcast_f(gap_v, rq), s_ttft = bcast_f(s_v, rq);
        const i64 off = (i64)bcast_u64((u64)off_v, rq);
        const u64 masks[5] = {bcast_u64(m_v[0], rq), bcast_u64(m_v[1], rq), bcast_u64(m_v[2], rq), bcast_u64(m_v[3], rq),
                              bcast_u64(m_v[4], rq)};
        const u64 dcol = (a.delivered != nullptr && !hist_pass) ? (1ull << a.delivered_col) : 0ull;
        TimelineResult res_lag{-1, 0.0f, 0};
        bool lag_done = false;
        // order buffer variants, lag, plain, device; a lag run that never fired is also the plain result
#pragma unroll 1
        for (int variant = 4; variant >= 0; --variant) {
            const u64 mask = variant == 4 ? masks[4] : (variant == 3 ? masks[3] : (variant == 2 ? masks[2] : (variant == 1 ? masks[1] : masks[0])));
            if (!mask) continue;
            float* deliv = (dcol & mask) ? a.delivered + off : nullptr;
            TimelineResult res;
            auto sink = [&](const unsigned key[4], const bool ok[4]) {
                if (hist_pass) hist_keys_cols(h, key, ok, mask, lane);
            };
            const bool src_dev = variant == 0 || variant == 4;
            const float gap = src_dev ? gd : gap_src;
            if (variant == 1 && lag_done && res_lag.m < 0 && !hist_pass && !deliv) {
                res = res_lag;
            } else if (variant < 3 && pure_pacing(src_dev || tr.arr == nullptr, gap, a.tau)) {
                res = run_pure_pacing(n, a.tau, lane, deliv, hist_pass, sink);
            } else {
                res = run_timeline(variant, n, tr.arr, off, n_tok, align, gap_src, gd, l, k, tr.c, s_ttft, a.bc, a.tau, a.kt,
                                   lane, deliv, sink);
            }
            if (variant == 2) { res_lag = res; lag_done = true; }
            if (hist_pass && a.pass == 0 && variant >= 3 && res.m >= 0 && ((mask >> lane) & 1ull)) {
                // lane = column: migrated requests by number of delayed tokens
                const int bin = res.delay < DISCO_DELAY_BINS - 1 ? res.delay : DISCO_DELAY_BINS - 1;
                atomicAdd(&a.dhist[(size_t)lane * DISCO_DELAY_BINS + bin], 1u);
            }
            if (!hist_pass && ((mask >> lane) & 1ull)) {
                const bool mig = res.m >= 0;
                const int nsrc = mig ? (variant >= 3 ? res.m + 1 : res.m) : n;      // tokens produced by the source
                if (src_dev) { acc_d_dec += (u64)nsrc; acc_s_dec += (u64)(n - nsrc); }
                else { acc_s_dec += (u64)nsrc; acc_d_dec += (u64)(n - nsrc); }
                if (mig) {
                    acc_mig += 1;
                    if (src_dev) acc_srepre += (u64)l + (u64)nsrc; else acc_repre += (u64)l + (u64)nsrc;
                    acc_delay += (u64)res.delay;
                }
                acc_cnt += (u64)(n - 1);
                acc_tlast += (double)res.t_last;
                if (a.mig_idx) a.mig_idx[(size_t)lane * tr.n_req + i] = mig ? nsrc : -1;
                if (a.n_src_tok) a.n_src_tok[(size_t)lane * tr.n_req + i] = nsrc;
                if (a.t_last) a.t_last[(size_t)lane * tr.n_req + i] = res.t_last;
                if (a.delay_num) a.delay_num[(size_t)lane * tr.n_req + i] = mig ? res.delay : 0;
            }
        }
      }
    }
    if (hist_pass) {
        __syncthreads();
        const int words = (P * nq) << h.width;
        for (int i = threadIdx.x; i < words; i += TL_BLOCK) {
            const unsigned cnt = smem[i];
            if (cnt) atomicAdd(&a.ghist[i], cnt);
        }
        return;
    }
    // statistics pass: fold the waves of the workgroup, then the workgroups (fixed order)
    u64* sh = reinterpret_cast<u64*>(smem);                                  // 8 fields x TL_BLOCK entries = 64 KB
    auto add = [](MigPartial& x, const MigPartial& o) {
        x.s_dec += o.s_dec; x.d_dec += o.d_dec; x.d_repre += o.d_repre; x.migrated += o.migrated;
        x.tbt_count += o.tbt_count; x.tlast_sum += o.tlast_sum; x.pad[0] += o.pad[0]; x.pad[1] += o.pad[1];
    };
    lds_put(sh, TL_BLOCK, wave * 64 + lane, MigPartial{acc_s_dec, acc_d_dec, acc_repre, acc_mig, acc_cnt, acc_tlast, {acc_srepre, acc_delay}});   // pad: server re-prefill, delayed tokens
    __syncthreads();
    if (threadIdx.x < 64) {
        MigPartial x = lds_get<MigPartial>(sh, TL_BLOCK, threadIdx.x);
        for (int w = 1; w < TL_WAVES; ++w) add(x, lds_get<MigPartial>(sh, TL_BLOCK, w * 64 + threadIdx.x));
        a.part[(size_t)bid * 64 + threadIdx.x] = x;
    }
    if (!take_last_ticket(a.ticket)) return;
    {
        const int c = threadIdx.x & 63, q = threadIdx.x >> 6;
        MigPartial x{0, 0, 0, 0, 0, 0.0, {0, 0}};
        for (unsigned b = q; b < nblk; b += TL_WAVES) add(x, a.part[(size_t)b * 64 + c]);
        __syncthreads();
        lds_put(sh, TL_BLOCK, q * 64 + c, x);
    }
    __syncthreads();
    if ((int)threadIdx.x < P) {
        const int c = threadIdx.x;
        MigPartial x = lds_get<MigPartial>(sh, TL_BLOCK, c);
        for (int q = 1; q < TL_WAVES; ++q) add(x, lds_get<MigPartial>(sh, TL_BLOCK, q * 64 + c));
        disco_accum* o = &a.acc[c];
        o->m_s_dec = (i64)x.s_dec; o->m_d_dec = (i64)x.d_dec; o->m_d_repre = (i64)x.d_repre;
        o->n_migrated = (i64)x.migrated; o->tbt_count = (i64)x.tbt_count; o->tlast_sum = x.tlast_sum;
        o->m_s_repre = (i64)x.pad[0]; o->delay_sum = (i64)x.pad[1];
    }
    if (threadIdx.x == 0) *a.ticket = 0u;
}

}  // namespace
