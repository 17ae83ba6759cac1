// One class-mode TBT histogram pass over the timelines of the streaming
// kinds (device source, server source, server source with the lag trigger;
// Sec. 4.3): the walker and the workgroup body, shared by the kernel of the
// regular passes and the kernel of the spare passes.
#pragma once
#include "disco_tl_walk.h"

namespace {

constexpr int TH_BLOCK = 1024;               // histogram workgroups: 16 waves share 64 KB of bins

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

// One histogram pass of the class-mode TBT selection, workgroup `bid` of `nblk`: the descriptors say which
// timelines have tokens to walk (few: the others were counted analytically once) and the walk list names their
// requests.  `smem`: DISCO_TL_HIST_WORDS words of LDS.
__device__ __forceinline__ void tl_hist_fast_body(unsigned* smem, const TraceView& tr, i64 n_tok, int align, const HistArgs& a,
                                                  unsigned bid, unsigned nblk)
{
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
    const i64 nwaves = (i64)nblk * (TH_BLOCK / 64);
    const i64 nfront = (i64)tl->nlist, nlist = nfront + (i64)tl->nlist_back;
    i64 rb = (nlist + nwaves - 1) / nwaves;
    rb = rb < 1 ? 1 : (rb > 64 ? 64 : rb);
    // wave w of a round takes the entries w, w + W, ... (lane = which of them), W = waves x rounds needed
    const i64 nround = (nlist + rb * nwaves - 1) / (rb * nwaves);
    for (i64 rnd = 0; rnd < nround; ++rnd) {
        const i64 gw = (i64)bid * (TH_BLOCK / 64) + wave;
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
