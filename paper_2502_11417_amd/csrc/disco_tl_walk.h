// Pieces shared by the kernels that walk token timelines in class mode: the
// per-request fields of a wave batch and the LDS histogram of the TBT
// selection (one row per class of timelines and prefix group).
#pragma once
#include "disco_tl_device.h"

namespace {

constexpr int TF_RB = 16;                    // requests per wave batch (at most; fewer on small traces, see tl_batch)
constexpr unsigned KEY_SKIP = 0x80000000u;   // a key with the sign bit never matches a prefix

// Per-request fields of a wave batch, lane = request (lanes >= TF_RB idle).
struct Batch {
    int l, n;
    float k, gd, gap, s;
    i64 off;
    u64 m[TL_KINDS];           // column sets by kind of timeline
};

__device__ __forceinline__ Batch load_batch(const TraceView& tr, const disco_policy* spol, int P, i64 first, int lane, int rb = TF_RB)
{
    Batch b;
    const i64 i = first + lane;
    const bool v = lane < rb && i < tr.n_req;
    b.l = 0; b.n = 1; b.k = tr.k_s; b.gd = tr.g_s; b.gap = 0.0f; b.off = 0; b.s = 0.0f;
    if (v) {
        b.l = tr.l[i]; b.n = tr.n[i]; b.s = tr.s[i];
        if (tr.k) b.k = tr.k[i];
        if (tr.g) b.gd = tr.g[i];
        if (tr.off) b.off = tr.off[i];
        if (tr.tbt) b.gap = tr.tbt[i];
    }
    request_sets(spol, P, b.l, b.s, __fmaf_rn((float)b.l, b.k, tr.c), i, b.m);
    if (!v) b.m[0] = b.m[1] = b.m[2] = b.m[3] = b.m[4] = 0ull;
    return b;
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
    int rb;                        // requests per wave batch
    SelState* S;
    unsigned* ghist;
    unsigned* ppcnt;
};

// Digit of this pass and the rows of the LDS histogram.
struct HistCtx {
    unsigned* hist;
    int shift, width, up, G;
    unsigned key_lo, key_cap;      // see tbt_key
    unsigned stride;               // words per prefix group = nwalk << width
    unsigned grp_prefix[DISCO_MAX_GRP];
};

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
