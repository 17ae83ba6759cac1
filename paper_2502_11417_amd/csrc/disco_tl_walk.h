// Pieces shared by the kernels that walk token timelines in class mode: the
// per-request fields of a wave batch and the LDS histogram of the TBT
// selection (one row per class of timelines and prefix group).
#pragma once
#include "disco_tl_device.h"

namespace {

constexpr int TF_RB = 16;                    // requests per wave batch (at most; fewer on small traces, see tl_batch)
constexpr unsigned KEY_SKIP = 0x80000000u;   // a key with the sign bit never matches a prefix

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

// Screening of the lag trigger (token t is overdue by more than kappa tau, Sec. 4.3 pacing) by a necessary
// condition.  With C <= M_{t-1} (C = a running maximum taken earlier, e.g. u_0) and monotone rounding,
//   lag_t = fl(r_t - fl(fl((t-1) tau + M_{t-1}) + tau)) <= fl(r_t - fl(fl((t-1) tau + C) + tau)),
// which differs from u_t - C = fl(r_t - t tau) - C by at most four roundings of magnitudes below
// 2 t tau + 2 |C| + kappa tau.  lag_fast_ok bounds t and the caller bounds |C| <= 2^18 kappa tau so that this
// error stays below kappa tau / 4; hence lag_t > kappa tau implies u_t > C + kappa tau / 2, and a chunk where
// no token satisfies the latter cannot trigger.
__device__ __forceinline__ bool lag_fast_ok(int n, float tau, float kt)
{
    return (float)n + 2.0f <= 262144.0f * (kt / tau) && kt >= tau * 0.0009765625f;
}

// What the token walk of disco_eval_migration leaves per request (16 bytes): the running maximum M = max_t u_t
// of each of its timelines that is not known in closed form -- the last delivery is fma(n-1, tau, M) -- and the
// lag hand-off.  Fields of kinds the request does not have, and of closed-form (pure-pacing) timelines, hold
// M = 0 and no hand-off, which is what such a timeline has.
//   M_lag    server source with the lag trigger (spliced device arrivals included)
//   m_enc    -1: no hand-off; -2: no hand-off and the first arrival offset is not 0; >= 0: first token produced
//            by the device in its low 30 bits, bit 30: the first arrival offset is not 0
//   M_plain  server source without hand-off
//   M_dev    device source
struct TlSummary { float M_lag; int m_enc; float M_plain; float M_dev; };
static_assert(sizeof(TlSummary) == 16, "one 16-byte store per request");

__device__ __forceinline__ int summary_m(int m_enc) { return m_enc < 0 ? -1 : (m_enc & 0x3FFFFFFF); }
__device__ __forceinline__ bool summary_r0_nonzero(int m_enc) { return m_enc == -2 || (m_enc >= 0 && ((m_enc >> 30) & 1)); }
// A server timeline whose running maximum never left its start 0: delta_t = round(t tau), like a pure-pacing
// constant-gap source; its gaps depend on its length alone.
__device__ __forceinline__ bool summary_pure_lag(const TlSummary& s) { return f2u(s.M_lag) == 0u && s.m_enc == -1; }
__device__ __forceinline__ bool summary_pure_plain(const TlSummary& s) { return f2u(s.M_plain) == 0u && !summary_r0_nonzero(s.m_enc); }

// Which walks a request needs (one byte per request, written before the walk): bit 0 server source with the
// lag trigger, bit 1 server source without hand-off, bit 2 device source; closed-form timelines need none.
// bit 3 (set by the streaming walk): its screening could not rule out a lag hand-off, the request is walked again, exactly.
enum { WF_LAG = 1, WF_PLAIN = 2, WF_DEV = 4, WF_REDO = 8 };

// Per-request fields of a wave batch, lane = request (lanes >= TF_RB idle).
struct Batch {
    int l, n;
    float k, gd, gap, s;
    i64 off;
    u64 m[TL_KINDS];           // column sets by kind of timeline
    TlSummary sum;             // what the token walk found (all zero / no hand-off without summaries)
};

// What the walk of the two buffer hand-off timelines of a request found (server source handed to the device,
// device source handed to the server): final running maximum, hand-off token in the encoding of
// TlSummary::m_enc (the source's last token), delayed tokens after the hand-off.
struct __attribute__((aligned(16))) BufSummary { float M_s; int m_s; int delay_s; int pad0; float M_d; int m_d; int delay_d; int pad1; };

__device__ __forceinline__ int buf_m_enc(int m, float r0)
{
    const bool nz = r0 != 0.0f;
    return m >= 0 ? (m | (nz ? (1 << 30) : 0)) : (nz ? -2 : -1);
}

// A buffer hand-off timeline whose running maximum never left 0 (first arrival 0 included) delivers token t at
// round(t tau) whatever its hand-off: histogrammed analytically like the pure-pacing timelines.
__device__ __forceinline__ bool buf_timeline_is_analytic(int kind, int n, const BufSummary& b)
{
    if (n < 0 || n > DISCO_PP_NMAX) return false;
    const float M = kind == TL_SRV_BUF ? b.M_s : b.M_d;
    const int me = kind == TL_SRV_BUF ? b.m_s : b.m_d;
    return f2u(M) == 0u && !summary_r0_nonzero(me);
}

// Is a timeline of kind TL_DEV, TL_SRV or TL_SRV_LAG histogrammed analytically?  Its running maximum never left 0
// and it has no hand-off, so delta_t = round(t tau) and its gaps depend on its length alone (counted per class
// and length up to DISCO_PP_NMAX).
__device__ __forceinline__ bool timeline_is_analytic(int kind, int n, const TlSummary& s)
{
    if (n < 0 || n > DISCO_PP_NMAX) return false;
    if (kind == TL_DEV) return f2u(s.M_dev) == 0u;
    return kind == TL_SRV ? summary_pure_plain(s) : summary_pure_lag(s);
}

__device__ __forceinline__ Batch load_batch(const TraceView& tr, const disco_policy* spol, int P, i64 first, int lane, int rb = TF_RB,
                                            const TlSummary* summary = nullptr)
{
    Batch b;
    b.sum = TlSummary{0.0f, -1, 0.0f, 0.0f};
    const i64 i = first + lane;
    const bool v = lane < rb && i < tr.n_req;
    b.l = 0; b.n = 1; b.k = tr.k_s; b.gd = tr.g_s; b.gap = 0.0f; b.off = 0; b.s = 0.0f;
    if (v) {
        b.l = tr.l[i]; b.n = tr.n[i]; b.s = tr.s[i];
        if (tr.k) b.k = tr.k[i];
        if (tr.g) b.gd = tr.g[i];
        if (tr.off) b.off = tr.off[i];
        if (tr.tbt) b.gap = tr.tbt[i];
        if (summary) b.sum = summary[i];
    }
    request_sets(spol, P, b.l, b.s, __fmaf_rn((float)b.l, b.k, tr.c), i, b.m);
    if (!v) b.m[0] = b.m[1] = b.m[2] = b.m[3] = b.m[4] = 0ull;
    return b;
}

// Totals of the timeline statistics -> accumulators (threads 0 .. P-1 of one workgroup, once every addition has
// been made); puts the totals back to zero for the next pass.
__device__ __forceinline__ void tl_stats_fin(int P, MigPartial* totals, disco_accum* acc)
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

// Requests a wave takes at a time: TF_RB on large traces; on small ones fewer, so that the waves the chip holds
// (`waves`) get several batches each and finish together.
inline int tl_batch(i64 n_req, i64 waves)
{
    int rb = TF_RB;
    while (rb > 1 && (n_req + rb - 1) / rb < 2 * waves) rb >>= 1;
    return rb;
}

struct HistArgs {
    float tau, kt;
    int P, pass;
    SelState* S;
    unsigned* ghist;
    const u64* desc;               // per request: LDS rows of its timelines that have tokens to walk (one byte per kind)
    const unsigned* list;          // requests with such a timeline (see walk_list_entry)
};

// Digit of this pass and the rows of the LDS histogram.
struct HistCtx {
    unsigned* hist;
    int shift, width, up, G;
    unsigned key_lo, key_cap;      // see tbt_key
    unsigned stride;               // words per prefix group = nwalk << width
    unsigned grp_prefix[DISCO_MAX_GRP];
};

// The walk list of the TBT selection: requests with 3 or more 256-token chunks are entered from the front, the
// others from the back of an array of `cap` slots.  The histogram kernels deal entry v to wave v mod W, so the long
// requests (which decide how long a pass takes) are spread evenly over the waves before the short ones fill in.
constexpr int WALK_LONG_TOKENS = 513;
__device__ __forceinline__ unsigned walk_list_entry(const unsigned* __restrict__ list, i64 cap, i64 nfront, i64 v)
{
    return v < nfront ? list[v] : list[cap - 1 - (v - nfront)];
}

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
        const unsigned kq = tbt_key(key[q], h.key_lo, h.key_cap);
        const unsigned hi = kq >> h.up;                          // the flag of skipped or clamped keys stays in
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
        idx[q] = g * h.stride + row_base + ((kq >> h.shift) & dmask);
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

}  // namespace
