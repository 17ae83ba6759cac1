// Token timelines (Sec. 4.3): paced delivery through the token buffer, the
// lag-triggered hand-off to the device, and the TBT histograms of the
// order-statistic selection.
//
// One wave walks one request at a time in chunks of 256 tokens, four
// consecutive tokens per lane (one 16-byte load per lane and chunk, the next
// chunk's load issued before the current one is used).  The delivery
// recurrence delta_t = max(r_t, delta_{t-1} + tau) is evaluated in the shifted
// domain u_t = r_t - t tau, where it is a running maximum: a 4-element scan in
// registers, a DPP scan across the wave, a carried maximum between chunks.
// `max` is exact and associative, so the result does not depend on the scan
// order and equals the sequential definition bit for bit.
//
// A timeline is computed once per request and source (server with hand-off,
// server without, device), never per policy column: the recurrence does not
// depend on the pair's TTFT, so every column only picks the timeline of its
// dispatch winner.  Lane j < P keeps column j's totals in registers.
#include <math.h>
#include <string.h>

#include "disco_launch.h"
#include "disco_state.h"

namespace {

// ---------------------------------------------------------------- scans ----

// dpp_ctrl encodings (GFX9): row_shr:n = 0x110 + n, wave_shr:1 = 0x138.
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float old, float src)
{
    return u2f((unsigned)__builtin_amdgcn_update_dpp((int)f2u(old), (int)f2u(src), CTRL, 0xF, 0xF, false));
}

// Inclusive running maximum over the 64 lanes: Hillis-Steele inside each row
// of 16 lanes with DPP row shifts (lanes whose source falls off the row keep
// -inf), then the three row totals are handed on through scalar registers.
__device__ __forceinline__ float wave_incl_max_dpp(float v, int lane)
{
    const float ninf = -INFINITY;
    v = fmaxf(v, dpp_mov<0x111>(ninf, v));
    v = fmaxf(v, dpp_mov<0x112>(ninf, v));
    v = fmaxf(v, dpp_mov<0x114>(ninf, v));
    v = fmaxf(v, dpp_mov<0x118>(ninf, v));
    const float t0 = bcast_f(v, 15), t1 = bcast_f(v, 31), t2 = bcast_f(v, 47);
    const float p1 = t0, p2 = fmaxf(t0, t1), p3 = fmaxf(p2, t2);
    const int row = lane >> 4;
    const float add = row == 0 ? ninf : (row == 1 ? p1 : (row == 2 ? p2 : p3));
    return fmaxf(v, add);
}

// Value of the previous lane (lane 0 receives `first`).
__device__ __forceinline__ float wave_prev(float v, float first)
{
    return dpp_mov<0x138>(first, v);
}

// ------------------------------------------------------------ histogram ----

// What a histogram pass needs, cached in LDS / registers per workgroup.
struct HistCtx {
    unsigned* hist;          // LDS bins
    int shift, width, up;    // digit of this pass; up = shift + width
    int fallback, ncls, G, nq;
    unsigned grp_prefix[DISCO_MAX_GRP];
    const u64* s_cls;        // LDS copy of the class table
    const unsigned* sprefix; // LDS, per slot (fallback path)
    const int* slive;        // LDS, per slot
};

// Class of a column set: index in the device-wide table, claimed on first use.
// Wave-uniform.  Returns -1 when the table is full.
__device__ __forceinline__ int cls_lookup(u64 mask, u64* s_cls, TlSel* tl, int lane)
{
    for (int attempt = 0; attempt < 2 * DISCO_MAX_CLS; ++attempt) {
        u64 m = s_cls[lane];
        u64 hit = __ballot(m == mask);
        if (hit) return __ffsll((long long)hit) - 1;
        m = __hip_atomic_load(&tl->cls_mask[lane], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        s_cls[lane] = m;
        hit = __ballot(m == mask);
        if (hit) return __ffsll((long long)hit) - 1;
        const u64 free = __ballot(m == 0ull);
        if (!free) return -1;
        const int e = __ffsll((long long)free) - 1;
        unsigned long long old = 0ull;
        if (lane == 0) old = atomicCAS((unsigned long long*)&tl->cls_mask[e], 0ull, (unsigned long long)mask);
        old = (unsigned long long)bcast_u64((u64)old, 0);
        if (old == 0ull || old == (unsigned long long)mask) {
            if (lane == 0) s_cls[e] = mask;
            return e;
        }
    }
    return -1;
}

// Class path: every key of the chunk goes to one histogram (prefix group g of
// the key, class c of the timeline).  The bin shared by most of the wave is
// counted with ballots and added once; the rest is added lane by lane.
__device__ __forceinline__ void hist_keys_cls(const HistCtx& h, const unsigned key[4], const bool ok[4], int cls, int lane)
{
    const unsigned dmask = (1u << h.width) - 1u;
    unsigned idx[4];
    bool pend[4];
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const unsigned hi = h.up >= 32 ? 0u : (key[q] >> h.up);
        int g = -1;
#pragma unroll
        for (int k = 0; k < DISCO_MAX_GRP; ++k) g = (k < h.G && hi == h.grp_prefix[k] && g < 0) ? k : g;
        pend[q] = ok[q] && g >= 0;
        idx[q] = ((unsigned)((g < 0 ? 0 : g) * h.ncls + cls) << h.width) | ((key[q] >> h.shift) & dmask);
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

// Fallback path: one histogram per (column, quantile) slot; a key counts for a
// slot if its upper bits equal the slot's prefix.  Columns that share a prefix
// are served together; equal bins are counted with ballots, lane = column adds.
__device__ __forceinline__ void hist_keys_cols(const HistCtx& h, const unsigned key[4], const bool ok[4], u64 cols, int lane)
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
                bin[k] = (key[k] >> h.shift) & dmask;
                pend[k] = ok[k] && ((h.up >= 32 ? 0u : (key[k] >> h.up)) == pf);
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

// Largest digit width whose `groups` histograms fit the LDS bins.
__device__ __host__ __forceinline__ int fit_width(int groups)
{
    int w = 0;
    while (w < 14 && ((size_t)groups << (w + 1)) <= (size_t)DISCO_TL_HIST_WORDS) ++w;
    return w;
}

// Prepares the next pass: prefix groups of the live slots, digit width that
// fits, or the per-slot fallback.  One thread.
__device__ void tbt_plan_next(SelState* S, int P, int nq)
{
    TlSel& tl = S->tl;
    int G = 0;
    bool over = tl.ncls > DISCO_MAX_CLS || tl.ncls < 1;
    for (int s = 0; s < P * nq; ++s) {
        const SelSlot sl = S->slot[1][s];
        int g = -1;
        if (!sl.done) {
            for (int k = 0; k < G && k < DISCO_MAX_GRP; ++k)
                if (tl.grp_prefix[k] == sl.prefix) g = k;
            if (g < 0) {
                if (G < DISCO_MAX_GRP) { tl.grp_prefix[G] = sl.prefix; g = G; }
                else g = 0;            // too many distinct prefixes: the per-slot fallback does not use groups
                G += 1;
            }
        }
        tl.slot_grp[s] = g;
    }
    if (G > DISCO_MAX_GRP) over = true;
    if (over) tl.fallback = 1;
    tl.G = G;
    int w = tl.fallback ? fit_width(P * nq) : fit_width((G > 0 ? G : 1) * tl.ncls);
    if (w < 1) w = 1;
    if (w > tl.left) w = tl.left;
    if (G == 0) w = 0;                 // nothing left to select
    tl.width = w;
    tl.shift = tl.left - w;
}

// After a TBT histogram pass: per live slot, add up the class histograms of
// the classes that contain the slot's column (or take the slot's own
// histogram in the fallback), walk to the digit that holds the remaining
// rank, extend the prefix; then plan the next pass and clear the bins.
__device__ void tbt_advance(SelState* S, int P, int nq, unsigned* ghist, const unsigned* ppcnt, float tau, unsigned* lds)
{
    TlSel& tl = S->tl;
    const int width = tl.width, ncls = tl.ncls, fallback = tl.fallback;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int Gused = tl.G < DISCO_MAX_GRP ? tl.G : DISCO_MAX_GRP;
    __syncthreads();
    if (width > 0 && !fallback) {
        // pure-pacing timelines: delta_t = round(t tau), so the gap in front of token t is the same for all
        // of them; ppcnt[c][t] timelines of class c have a token t.  Bins are gathered in LDS first.
        const int words = (Gused * ncls) << width;
        const int shift = tl.shift, up = tl.shift + width;
        const unsigned dmask = (1u << width) - 1u;
        for (int i = threadIdx.x; i < words; i += blockDim.x) lds[i] = 0u;
        __syncthreads();
        for (int t = 1 + (int)threadIdx.x; t < DISCO_PP_NMAX; t += blockDim.x) {
            const unsigned key = f2u((float)t * tau - (float)(t - 1) * tau);
            const unsigned hi = up >= 32 ? 0u : (key >> up);
            int g = -1;
            for (int k = 0; k < Gused; ++k) g = (hi == tl.grp_prefix[k] && g < 0) ? k : g;
            if (g < 0) continue;
            for (int c = 0; c < ncls; ++c) {
                const unsigned cnt = ppcnt[(size_t)c * (DISCO_PP_NMAX + 1) + t];
                if (cnt) atomicAdd(&lds[((unsigned)(g * ncls + c) << width) | ((key >> shift) & dmask)], cnt);
            }
        }
        __syncthreads();
        for (int i = threadIdx.x; i < words; i += blockDim.x) ghist[i] += lds[i];
        __threadfence_block();
        __syncthreads();
    }
    if (width > 0) {
        const int nbins = 1 << width;
        const int per = (nbins + 63) >> 6;
        for (int s = wave; s < P * nq; s += nwaves) {
            SelSlot sl = S->slot[1][s];
            const int g = tl.slot_grp[s];
            if (sl.done || g < 0) continue;
            const int col = s / nq;
            const int b0 = lane * per;
            auto bin_count = [&](int b) -> u64 {
                if (fallback) return ghist[((size_t)s << width) | b];
                u64 c = 0;
                for (int k = 0; k < ncls; ++k)
                    if ((tl.cls_mask[k] >> col) & 1ull) c += ghist[((size_t)(g * ncls + k) << width) | b];
                return c;
            };
            u64 mine = 0;
            for (int b = b0; b < b0 + per && b < nbins; ++b) mine += bin_count(b);
            u64 incl = mine;
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                unsigned lo = (unsigned)__shfl_up((int)(unsigned)incl, d, 64);
                unsigned hi = (unsigned)__shfl_up((int)(unsigned)(incl >> 32), d, 64);
                if (lane >= d) incl += ((u64)hi << 32) | lo;
            }
            const u64 k = (u64)sl.k_rem;
            const u64 hit = __ballot(incl >= k);
            const int owner = hit ? (__ffsll((long long)hit) - 1) : 63;
            if (lane == owner) {
                u64 rem = k - (incl - mine);
                int dsel = nbins - 1;
                for (int b = b0; b < b0 + per && b < nbins; ++b) {
                    const u64 c = bin_count(b);
                    if (rem <= c) { dsel = b; break; }
                    rem -= c;
                }
                sl.k_rem = (i64)rem;
                sl.prefix = (sl.prefix << width) | (unsigned)dsel;
                S->slot[1][s] = sl;
            }
        }
    }
    __syncthreads();
    if (width > 0) {
        const int words = (fallback ? P * nq : Gused * ncls) << width;
        for (int i = threadIdx.x; i < words; i += blockDim.x) ghist[i] = 0u;
    }
    __threadfence_block();
    __syncthreads();
    if (threadIdx.x == 0) {
        tl.left -= width;
        if (tl.left <= 0) { tl.left = 0; tl.width = 0; tl.G = 0; }
        else tbt_plan_next(S, P, nq);
    }
}

// ------------------------------------------------------------- timeline ----

struct TimelineResult { int m; float t_last; };

// Loads the four arrival offsets of this lane for the chunk that starts at
// element index `e0` of the request's (aligned) token window.
//   g      global index of the lane's first element, may lie outside [0, n_tok)
__device__ __forceinline__ void load4(const float* __restrict__ arr, i64 g, i64 n_tok, float r[4])
{
    if (g >= 0 && g + 3 < n_tok) {
        const float4 v = *reinterpret_cast<const float4*>(arr + g);
        r[0] = v.x; r[1] = v.y; r[2] = v.z; r[3] = v.w;
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) r[k] = (g + k >= 0 && g + k < n_tok) ? arr[g + k] : 0.0f;
    }
}

// Timeline of one request and source.
//   variant 0: device source, 1: server source, 2: server source with the lag trigger
//   arr/off/n_tok: CSR token array or arr == nullptr (constant gap `gap_src`)
//   deliv: nullable, delivery offsets of the request's tokens
//   sink(key[4], ok[4]): called once per chunk by all lanes (ok marks real gaps)
template <class Sink>
__device__ __forceinline__ TimelineResult run_timeline(int variant, int n, const float* __restrict__ arr, i64 off, i64 n_tok,
                                                       int align, float gap_src, float g_dev, int l, float k, float c,
                                                       float tau, float kt, int lane, float* __restrict__ deliv, Sink&& sink)
{
    const bool from_mem = (variant != 0) && arr != nullptr;
    const float gap = (variant == 0) ? g_dev : gap_src;
    // element 0 of the window is the aligned-down start: the first `mis` elements precede the request
    const int mis = from_mem ? (int)((off + align) & 3) : 0;
    const i64 gbase = off - mis + 4 * lane;
    float carryM = -INFINITY, carryD = INFINITY, base = 0.0f, t_last = 0.0f;
    int m = -1;
    float nxt[4] = {0.f, 0.f, 0.f, 0.f};
    if (from_mem && 4 * lane - mis < n) load4(arr, gbase, n_tok, nxt);
    const int total = n + mis;
    for (int e0 = 0; e0 < total; e0 += 256) {
        const int tb = e0 + 4 * lane - mis;                 // token index of this lane's first element
        float r[4];
        int tk[4];
        float tf[4];
        bool val[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) { tk[q] = tb + q; tf[q] = (float)tk[q]; val[q] = tk[q] >= 0 && tk[q] < n; }
        if (from_mem && m < 0) {
#pragma unroll
            for (int q = 0; q < 4; ++q) r[q] = nxt[q];
            if (e0 + 256 < total && tb + 256 < n) load4(arr, gbase + e0 + 256, n_tok, nxt);   // next chunk in flight
        } else if (m < 0) {
#pragma unroll
            for (int q = 0; q < 4; ++q) r[q] = tf[q] * gap;
        }
        if (m >= 0) {
#pragma unroll
            for (int q = 0; q < 4; ++q) r[q] = __fmaf_rn((float)(tk[q] - m + 1), g_dev, base);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) r[q] = val[q] ? r[q] : -INFINITY;
        float d[4], prev[4];
        float Mlast;
        auto scan = [&]() {
            float u[4], mx[4];
#pragma unroll
            for (int q = 0; q < 4; ++q) u[q] = __fmaf_rn(-tf[q], tau, r[q]);      // -inf for lanes outside the request
            mx[0] = u[0]; mx[1] = fmaxf(mx[0], u[1]); mx[2] = fmaxf(mx[1], u[2]); mx[3] = fmaxf(mx[2], u[3]);
            const float incl = wave_incl_max_dpp(mx[3], lane);
            const float excl = fmaxf(wave_prev(incl, -INFINITY), carryM);
#pragma unroll
            for (int q = 0; q < 4; ++q) d[q] = __fmaf_rn(tf[q], tau, fmaxf(excl, mx[q]));
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
                    if (tk[q] >= m) r[q] = val[q] ? __fmaf_rn((float)(tk[q] - m + 1), g_dev, base) : -INFINITY;
                scan();
            }
        }
        unsigned key[4];
        bool ok[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            key[q] = f2u(d[q] - prev[q]);
            ok[q] = val[q] && tk[q] >= 1;
            if (deliv && val[q]) deliv[tk[q]] = d[q];
        }
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
    return TimelineResult{m, t_last};
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
    return TimelineResult{-1, (float)(n - 1) * tau};
}

constexpr int TL_BLOCK = 1024;
constexpr int TL_WAVES = TL_BLOCK / 64;
constexpr int TL_RB = 16;                   // requests per wave batch
constexpr int TL_HIST_WORDS = 16384;        // 64 KB of LDS histogram: two workgroups per CU

__global__ __launch_bounds__(TL_BLOCK, 2) void k_timeline(TraceView tr, i64 n_tok, int align,
                                                       const disco_policy* __restrict__ pol, TimelineArgs a)
{
    __shared__ __align__(16) unsigned smem[TL_HIST_WORDS];
    __shared__ unsigned sprefix[DISCO_MAX_SLOTS];
    __shared__ int slive[DISCO_MAX_SLOTS];
    __shared__ u64 s_cls[DISCO_MAX_CLS];
    __shared__ disco_policy spol[DISCO_MAX_COLS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int P = a.P, nq = a.nq;
    if ((int)threadIdx.x < P) spol[threadIdx.x] = pol[threadIdx.x];
    const bool hist_pass = a.pass >= 0;       // pass -1: statistics
    const bool classify = false;
    HistCtx h;
    h.hist = smem; h.shift = 0; h.width = 0; h.up = 0; h.fallback = 0; h.ncls = 1; h.G = 0; h.nq = nq;
    h.s_cls = s_cls; h.sprefix = sprefix; h.slive = slive;
    for (int k = 0; k < DISCO_MAX_GRP; ++k) h.grp_prefix[k] = 0u;
    if (hist_pass || classify) {
        TlSel* tl = &a.S->tl;
        if (threadIdx.x < DISCO_MAX_CLS)
            s_cls[threadIdx.x] = __hip_atomic_load(&tl->cls_mask[threadIdx.x], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (hist_pass) {
        const TlSel* tl = &a.S->tl;
        h.width = tl->width;
        if (h.width <= 0) return;             // selection finished: nothing to do in this launch
        h.shift = tl->shift;
        h.up = h.shift + h.width;
        h.fallback = tl->fallback; h.ncls = tl->ncls; h.G = tl->G < DISCO_MAX_GRP ? tl->G : DISCO_MAX_GRP;
        for (int k = 0; k < DISCO_MAX_GRP; ++k) h.grp_prefix[k] = tl->grp_prefix[k];
        const int words = (h.fallback ? P * nq : h.G * h.ncls) << h.width;
        for (int i = threadIdx.x; i < words; i += TL_BLOCK) smem[i] = 0u;
        for (int i = threadIdx.x; i < P * nq; i += TL_BLOCK) {
            const SelSlot sl = a.S->slot[1][i];
            sprefix[i] = sl.prefix;
            slive[i] = !sl.done;
        }
    }
    __syncthreads();
    const bool work = true;
    u64 acc_s_dec = 0, acc_d_dec = 0, acc_repre = 0, acc_mig = 0, acc_cnt = 0;
    double acc_tlast = 0.0;
    const i64 nwaves = (i64)gridDim.x * TL_WAVES;
    // A wave takes TL_RB consecutive requests at a time.  Phase A, lane = request: the fields are
    // loaded coalesced and every column's dispatch is evaluated, giving the three column sets of the
    // request (device source, server source, server source with lag hand-off).  Phase B walks the
    // requests one by one with the whole wave on the tokens.
    const i64 nbatch = (tr.n_req + TL_RB - 1) / TL_RB;
    for (i64 bt = (i64)blockIdx.x * TL_WAVES + wave; work && bt < nbatch; bt += nwaves) {
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
        u64 m_v[3] = {0ull, 0ull, 0ull};
        {
            const float d_v = __fmaf_rn((float)l_v, k_v, tr.c);
            for (int j = 0; j < P; ++j) {
                unsigned dec; float t;
                dispatch_pair(spol[j], l_v, s_v, d_v, dec, t);
                const int kind = (dec & 4u) ? 0 : (spol[j].mig_mode == DISCO_MIG_LAG ? 2 : 1);
                m_v[kind] |= va ? (1ull << j) : 0ull;
            }
        }
        const int cnt = (int)((tr.n_req - bt * TL_RB < TL_RB) ? (tr.n_req - bt * TL_RB) : TL_RB);
#pragma unroll 1
      for (int rq = 0; rq < cnt; ++rq) {
        const i64 i = bt * TL_RB + rq;
        const int l = bcast_i(l_v, rq), n = bcast_i(n_v, rq);
        const float k = bcast_f(k_v, rq), gd = bcast_f(g_v, rq);
        const float gap_src = bcast_f(gap_v, rq);
        const i64 off = (i64)bcast_u64((u64)off_v, rq);
        const u64 mask_dev = bcast_u64(m_v[0], rq), mask_plain = bcast_u64(m_v[1], rq), mask_lag = bcast_u64(m_v[2], rq);
        const u64 dcol = (a.delivered != nullptr && !hist_pass) ? (1ull << a.delivered_col) : 0ull;
        TimelineResult res_lag{-1, 0.0f};
        bool lag_done = false;
        // order lag, plain, device; a lag run that never fired is also the plain result
#pragma unroll 1
        for (int variant = 2; variant >= 0; --variant) {
            const u64 mask = variant == 2 ? mask_lag : (variant == 1 ? mask_plain : mask_dev);
            if (!mask) continue;
            float* deliv = (dcol & mask) ? a.delivered + off : nullptr;
            TimelineResult res;
            int cls = 0;
            if (classify || (hist_pass && !h.fallback)) {
                cls = cls_lookup(mask, s_cls, &a.S->tl, lane);
                if (cls < 0) {                      // table full: the selection falls back to per-column histograms
                    if (lane == 0) a.S->tl.error = 1;
                    cls = 0;
                }
            }
            if (classify) continue;
            auto sink = [&](const unsigned key[4], const bool ok[4]) {
                if (!hist_pass) return;
                if (h.fallback) hist_keys_cols(h, key, ok, mask, lane);
                else hist_keys_cls(h, key, ok, cls, lane);
            };
            const float gap = variant == 0 ? gd : gap_src;
            const bool constant = variant == 0 || tr.arr == nullptr;
            if (variant == 1 && lag_done && res_lag.m < 0 && !hist_pass && !deliv) {
                res = res_lag;
            } else if (constant && gap < 0.999f * a.tau) {
                // in a class-mode histogram pass the bins of short pure-pacing timelines are filled analytically
                const bool walk = hist_pass && (h.fallback || n > DISCO_PP_NMAX);
                res = run_pure_pacing(n, a.tau, lane, deliv, walk, sink);
            } else {
                res = run_timeline(variant, n, tr.arr, off, n_tok, align, gap_src, gd, l, k, tr.c, a.tau, a.kt, lane,
                                   deliv, sink);
            }
            if (variant == 2) { res_lag = res; lag_done = true; }
            if (!hist_pass && ((mask >> lane) & 1ull)) {
                const int nsrc = (res.m >= 0) ? res.m : n;
                if (variant == 0) acc_d_dec += (u64)n;
                else { acc_s_dec += (u64)nsrc; acc_d_dec += (u64)(n - nsrc); }
                if (res.m >= 0) { acc_mig += 1; acc_repre += (u64)l + (u64)res.m; }
                acc_cnt += (u64)(n - 1);
                acc_tlast += (double)res.t_last;
                if (a.mig_idx) a.mig_idx[(size_t)lane * tr.n_req + i] = res.m;
                if (a.n_src_tok) a.n_src_tok[(size_t)lane * tr.n_req + i] = nsrc;
                if (a.t_last) a.t_last[(size_t)lane * tr.n_req + i] = res.t_last;
            }
        }
      }
    }
    if (hist_pass) {
        __syncthreads();
        const int words = (h.fallback ? P * nq : h.G * h.ncls) << h.width;
        for (int i = threadIdx.x; i < words; i += TL_BLOCK) {
            const unsigned cnt = smem[i];
            if (cnt) atomicAdd(&a.ghist[i], cnt);
        }
        if (!take_last_ticket(a.ticket)) return;
        tbt_advance(a.S, P, nq, a.ghist, a.ppcnt, a.tau, smem);
        if (threadIdx.x == 0) *a.ticket = 0u;
        return;
    }
    // statistics pass: fold the waves of the workgroup, then the workgroups (fixed order)
    u64* sh = reinterpret_cast<u64*>(smem);                                  // 8 fields x TL_BLOCK entries = 64 KB
    auto add = [](MigPartial& x, const MigPartial& o) {
        x.s_dec += o.s_dec; x.d_dec += o.d_dec; x.d_repre += o.d_repre; x.migrated += o.migrated;
        x.tbt_count += o.tbt_count; x.tlast_sum += o.tlast_sum;
    };
    lds_put(sh, TL_BLOCK, wave * 64 + lane, MigPartial{acc_s_dec, acc_d_dec, acc_repre, acc_mig, acc_cnt, acc_tlast, {0, 0}});
    __syncthreads();
    if (threadIdx.x < 64) {
        MigPartial x = lds_get<MigPartial>(sh, TL_BLOCK, threadIdx.x);
        for (int w = 1; w < TL_WAVES; ++w) add(x, lds_get<MigPartial>(sh, TL_BLOCK, w * 64 + threadIdx.x));
        a.part[(size_t)blockIdx.x * 64 + threadIdx.x] = x;
    }
    if (!take_last_ticket(a.ticket)) return;
    {
        const int c = threadIdx.x & 63, q = threadIdx.x >> 6;
        MigPartial x{0, 0, 0, 0, 0, 0.0, {0, 0}};
        for (unsigned b = q; b < gridDim.x; b += TL_WAVES) add(x, a.part[(size_t)b * 64 + c]);
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
    }
    if (threadIdx.x == 0) *a.ticket = 0u;
}

// The three column sets of a request, lane = request.
__device__ __forceinline__ void request_sets(const TraceView& tr, const disco_policy* sp, int P, i64 i, bool v, u64 m[3],
                                             int& n, float& gd, float& gap)
{
    m[0] = m[1] = m[2] = 0ull;
    n = 1; gd = tr.g_s; gap = 0.0f;
    if (!v) return;
    const int l = tr.l[i];
    const float s = tr.s[i];
    const float k = tr.k ? tr.k[i] : tr.k_s;
    const float d = __fmaf_rn((float)l, k, tr.c);
    n = tr.n[i];
    if (tr.g) gd = tr.g[i];
    if (tr.tbt) gap = tr.tbt[i];
    for (int j = 0; j < P; ++j) {
        unsigned dec; float t;
        dispatch_pair(sp[j], l, s, d, dec, t);
        const int kind = (dec & 4u) ? 0 : (sp[j].mig_mode == DISCO_MIG_LAG ? 2 : 1);
        m[kind] |= 1ull << j;
    }
}

// Column sets of every request -> classes.  The distinct sets of a workgroup
// are first collected in LDS and then claimed in the device-wide table by one
// wave, so the few hot table lines are touched once per workgroup; the last
// workgroup plans the first histogram pass.  Also clears the length counts.
__global__ __launch_bounds__(256) void k_tl_classify(TraceView tr, const disco_policy* __restrict__ pol, int P, int nq,
                                                     SelState* S, unsigned* ppcnt, unsigned* ticket)
{
    __shared__ disco_policy sp[DISCO_MAX_COLS];
    __shared__ u64 loc[DISCO_MAX_CLS];
    __shared__ u64 s_cls[DISCO_MAX_CLS];
    __shared__ int overflow;
    if ((int)threadIdx.x < P) sp[threadIdx.x] = pol[threadIdx.x];
    if (threadIdx.x < DISCO_MAX_CLS) { loc[threadIdx.x] = 0ull; s_cls[threadIdx.x] = 0ull; }
    if (threadIdx.x == 0) overflow = 0;
    for (i64 w = (i64)blockIdx.x * 256 + threadIdx.x; w < (i64)DISCO_MAX_CLS * (DISCO_PP_NMAX + 1); w += (i64)gridDim.x * 256)
        ppcnt[w] = 0u;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    const i64 nround = (tr.n_req + 255) / 256;
    for (i64 rnd = blockIdx.x; rnd < nround; rnd += gridDim.x) {
        const i64 i = rnd * 256 + threadIdx.x;
        u64 m[3];
        int n; float gd, gap;
        request_sets(tr, sp, P, i, i < tr.n_req, m, n, gd, gap);
#pragma unroll
        for (int kind = 0; kind < 3; ++kind) {
            u64 pend = __ballot(m[kind] != 0ull);
            while (pend) {
                const int leader = __ffsll((long long)pend) - 1;
                const u64 m0 = bcast_u64(m[kind], leader);
                pend &= ~__ballot(m[kind] == m0);
                for (int attempt = 0; attempt < DISCO_MAX_CLS + 1; ++attempt) {     // insert m0 into the workgroup's table
                    const u64 cur = loc[lane];
                    if (__ballot(cur == m0)) break;
                    const u64 free = __ballot(cur == 0ull);
                    if (!free) { if (lane == 0) overflow = 1; break; }
                    const int e = __ffsll((long long)free) - 1;
                    if (lane == 0) atomicCAS((unsigned long long*)&loc[e], 0ull, (unsigned long long)m0);
                }
            }
        }
    }
    __syncthreads();
    if (threadIdx.x < 64) {
        u64 mine = __ballot(loc[lane] != 0ull);
        bool bad = overflow != 0;
        while (mine) {
            const int e = __ffsll((long long)mine) - 1;
            mine &= mine - 1;
            if (cls_lookup(loc[e], s_cls, &S->tl, lane) < 0) bad = true;
        }
        if (bad && lane == 0) S->tl.error = 1;
    }
    if (!take_last_ticket(ticket)) return;
    if (threadIdx.x == 0) {
        TlSel& tl = S->tl;
        int n = 0;
        for (int k = 0; k < DISCO_MAX_CLS; ++k)
            if (__hip_atomic_load(&tl.cls_mask[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0ull) n = k + 1;
        tl.ncls = n > 0 ? n : 1;
        if (__hip_atomic_load(&tl.error, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT)) { tl.fallback = 1; tl.error = 0; }
        tl.left = 31;
        tbt_plan_next(S, P, nq);
        *ticket = 0u;
    }
}

// Is the timeline of this kind pure pacing (see run_pure_pacing) and short
// enough for the analytic histogram?
__device__ __forceinline__ bool analytic_kind(const TraceView& tr, int kind, int n, float gd, float gap, float tau)
{
    const bool constant = kind == 0 || tr.arr == nullptr;
    const float gp = kind == 0 ? gd : gap;
    return constant && gp < 0.999f * tau && n <= DISCO_PP_NMAX;
}

// Pure-pacing timelines depend on their length alone: count them per class
// and length instead of walking their tokens in every histogram pass.
__global__ __launch_bounds__(256) void k_pp_count(TraceView tr, const disco_policy* __restrict__ pol, int P, float tau,
                                                  SelState* S, unsigned* ppcnt)
{
    __shared__ disco_policy sp[DISCO_MAX_COLS];
    __shared__ u64 s_cls[DISCO_MAX_CLS];
    if (S->tl.fallback) return;
    if ((int)threadIdx.x < P) sp[threadIdx.x] = pol[threadIdx.x];
    if (threadIdx.x < DISCO_MAX_CLS) s_cls[threadIdx.x] = S->tl.cls_mask[threadIdx.x];
    __syncthreads();
    for (i64 i = (i64)blockIdx.x * 256 + threadIdx.x; i < tr.n_req; i += (i64)gridDim.x * 256) {
        u64 m[3];
        int n; float gd, gap;
        request_sets(tr, sp, P, i, true, m, n, gd, gap);
#pragma unroll
        for (int kind = 0; kind < 3; ++kind) {
            if (m[kind] == 0ull || !analytic_kind(tr, kind, n, gd, gap, tau)) continue;
            int c = -1;
            for (int k = 0; k < DISCO_MAX_CLS; ++k) c = (s_cls[k] == m[kind]) ? k : c;
            if (c >= 0) atomicAdd(&ppcnt[(size_t)c * (DISCO_PP_NMAX + 1) + n], 1u);
            else S->tl.error = 1;          // a set the classification did not see: never expected
        }
    }
}

// Per class: counts by length -> number of timelines longer than t (in place).
__global__ __launch_bounds__(1024) void k_pp_suffix(SelState* S, unsigned* ppcnt)
{
    __shared__ unsigned part[1024];
    if (S->tl.fallback || (int)blockIdx.x >= S->tl.ncls) return;
    unsigned* row = ppcnt + (size_t)blockIdx.x * (DISCO_PP_NMAX + 1);
    constexpr int PER = (DISCO_PP_NMAX + 1 + 1023) / 1024;
    const int t0 = threadIdx.x * PER;
    unsigned v[PER];
    unsigned sum = 0;
    for (int q = 0; q < PER; ++q) { v[q] = (t0 + q <= DISCO_PP_NMAX) ? row[t0 + q] : 0u; sum += v[q]; }
    part[threadIdx.x] = sum;
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {            // inclusive suffix sums of the per-thread totals
        const unsigned o = (threadIdx.x + d < 1024) ? part[threadIdx.x + d] : 0u;
        __syncthreads();
        part[threadIdx.x] += o;
        __syncthreads();
    }
    unsigned above = (threadIdx.x + 1 < 1024) ? part[threadIdx.x + 1] : 0u;       // lengths beyond this thread's slice
    for (int q = PER - 1; q >= 0; --q) {
        if (t0 + q <= DISCO_PP_NMAX) row[t0 + q] = above;                         // timelines with n > t0 + q
        above += v[q];
    }
}

}  // namespace

void disco_launch_tl_prepare(const TraceView& v, const disco_policy* pol, int P, int nq, float tau, SelState* S,
                             unsigned* ppcnt, unsigned* ticket, hipStream_t stream)
{
    i64 b = (v.n_req + 255) / 256;
    if (b < 1) b = 1;
    if (b > 512) b = 512;
    hipLaunchKernelGGL(k_tl_classify, dim3((unsigned)b), dim3(256), 0, stream, v, pol, P, nq, S, ppcnt, ticket);
    hipLaunchKernelGGL(k_pp_count, dim3((unsigned)b), dim3(256), 0, stream, v, pol, P, tau, S, ppcnt);
    hipLaunchKernelGGL(k_pp_suffix, dim3(DISCO_MAX_CLS), dim3(1024), 0, stream, S, ppcnt);
}

void disco_launch_timeline(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a, hipStream_t stream)
{
    i64 b = (v.n_req + (i64)TL_WAVES * TL_RB - 1) / ((i64)TL_WAVES * TL_RB);
    if (b < 1) b = 1;
    if (b > 512) b = 512;                     // two resident workgroups per CU
    const int align = (int)(((uintptr_t)v.arr >> 2) & 3);
    hipLaunchKernelGGL(k_timeline, dim3((unsigned)b), dim3(TL_BLOCK), 0, stream, v, n_tok, align, pol, a);
}
