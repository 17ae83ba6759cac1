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
__device__ void tbt_advance(SelState* S, int P, int nq, unsigned* ghist)
{
    TlSel& tl = S->tl;
    const int width = tl.width, ncls = tl.ncls, fallback = tl.fallback;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, nwaves = blockDim.x >> 6;
    const int Gused = tl.G < DISCO_MAX_GRP ? tl.G : DISCO_MAX_GRP;
    __syncthreads();
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

constexpr int TL_BLOCK = 512;
constexpr int TL_WAVES = TL_BLOCK / 64;
constexpr int TL_HIST_WORDS = 16384;        // 64 KB of LDS histogram: two workgroups per CU

__global__ __launch_bounds__(TL_BLOCK) void k_timeline(TraceView tr, i64 n_tok, int align,
                                                       const disco_policy* __restrict__ pol, TimelineArgs a)
{
    __shared__ __align__(16) unsigned smem[TL_HIST_WORDS];
    __shared__ unsigned sprefix[DISCO_MAX_SLOTS];
    __shared__ int slive[DISCO_MAX_SLOTS];
    __shared__ u64 s_cls[DISCO_MAX_CLS];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int P = a.P, nq = a.nq;
    const bool colv = lane < P;
    const disco_policy p = pol[colv ? lane : 0];
    const bool hist_pass = a.pass >= 0;       // pass -1: statistics, -2: classification of the column sets
    const bool classify = a.pass == -2;
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
    for (i64 i = (i64)blockIdx.x * TL_WAVES + wave; work && i < tr.n_req; i += nwaves) {
        const int l = tr.l[i], n = tr.n[i];
        const float s = tr.s[i];
        const float k = tr.k ? tr.k[i] : tr.k_s;
        const float gd = tr.g ? tr.g[i] : tr.g_s;
        const float d = __fmaf_rn((float)l, k, tr.c);
        unsigned dec; float ttft;
        dispatch_pair(p, l, s, d, dec, ttft);
        const bool dev_src = (dec & 4u) != 0u;
        const u64 mask_dev = __ballot(colv && dev_src);
        const u64 mask_plain = __ballot(colv && !dev_src && p.mig_mode != DISCO_MIG_LAG);
        const u64 mask_lag = __ballot(colv && !dev_src && p.mig_mode == DISCO_MIG_LAG);
        const i64 off = tr.off ? tr.off[i] : 0;
        const float gap_src = tr.tbt ? tr.tbt[i] : 0.0f;
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
                res = run_pure_pacing(n, a.tau, lane, deliv, hist_pass, sink);
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
    if (classify) {
        if (!take_last_ticket(a.ticket)) return;
        if (threadIdx.x == 0) {                     // all column sets are known: plan the first histogram pass
            TlSel& tl = a.S->tl;
            int n = 0;
            for (int k = 0; k < DISCO_MAX_CLS; ++k)
                if (__hip_atomic_load(&tl.cls_mask[k], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0ull) n = k + 1;
            tl.ncls = n > 0 ? n : 1;
            if (tl.error) { tl.fallback = 1; tl.error = 0; }
            tl.left = 31;
            tbt_plan_next(a.S, P, nq);
            *a.ticket = 0u;
        }
        return;
    }
    if (hist_pass) {
        __syncthreads();
        const int words = (h.fallback ? P * nq : h.G * h.ncls) << h.width;
        for (int i = threadIdx.x; i < words; i += TL_BLOCK) {
            const unsigned cnt = smem[i];
            if (cnt) atomicAdd(&a.ghist[i], cnt);
        }
        if (!take_last_ticket(a.ticket)) return;
        tbt_advance(a.S, P, nq, a.ghist);
        if (threadIdx.x == 0) *a.ticket = 0u;
        return;
    }
    // statistics pass: fold the waves of the workgroup, then the workgroups (fixed order)
    u64* sh = reinterpret_cast<u64*>(smem);                                  // 8 fields x TL_BLOCK entries = 32 KB
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

}  // namespace

void disco_launch_timeline(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a, hipStream_t stream)
{
    i64 b = (v.n_req + TL_WAVES - 1) / TL_WAVES;
    if (b < 1) b = 1;
    if (b > 512) b = 512;                     // two resident workgroups per CU
    const int align = (int)(((uintptr_t)v.arr >> 2) & 3);
    hipLaunchKernelGGL(k_timeline, dim3((unsigned)b), dim3(TL_BLOCK), 0, stream, v, n_tok, align, pol, a);
}
