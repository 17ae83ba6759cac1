// TBT order statistics over token timelines (Sec. 5.1 metrics on the
// timelines of Sec. 4.3): classes of timelines, analytic histogram of
// pure-pacing timelines, digit selection between the histogram passes.
//
// A timeline is histogrammed once per class = set of policy columns that use
// it, not once per column.  For threshold- or wait-ordered tables the sets
// are nested, so there are at most P + 1 of them per source.  Classes whose
// members are all short pure-pacing timelines (constant source gap below the
// pacing interval) need no token walk at all: the gap in front of token t is
// round(t tau) - round((t-1) tau) for every one of them, so counting the
// timelines per class and length gives their histogram.
//
// Launches of a selection: classification, assignment (other file), the
// "longer than" counts; per regular pass the walk of the streaming kinds
// (other file), k_tbt_side (analytic bins, buffer hand-off timelines,
// per-slot histograms: workgroups by kind) and k_tbt_select (one workgroup
// per slot; the last one plans the next pass); per spare pass k_tbt_spare
// alone.  A launch that finds the selection finished returns at once, which
// still costs about 2 us on the device: hence few launches.
#include <string.h>

#include "disco_tl_general_kernel.h"
#include "disco_tl_hist_buf.h"
#include "disco_tl_hist_fast.h"

namespace {

// Prepares the next pass: prefix groups of the live slots, digit width that
// fits, or the per-slot fallback.  All threads of a workgroup (wave_only: of
// its first wave, the only one still running); the slots are fetched side by
// side into LDS (s_prefix, s_grp: DISCO_MAX_SLOTS words each), one thread
// groups them there.  reset: every slot starts over (empty prefix, full rank).
__device__ void tbt_plan_next(SelState* S, int P, int nq, unsigned* s_prefix, int* s_grp, bool wave_only, bool reset)
{
    TlSel& tl = S->tl;
    const int ns = P * nq, nt = wave_only ? 64 : (int)blockDim.x;
    auto sync = [&]() { if (wave_only) __builtin_amdgcn_wave_barrier(); else __syncthreads(); };
    for (int s = threadIdx.x; s < ns; s += nt) {
        SelSlot sl = S->slot[1][s];
        if (reset) { sl.prefix = 0u; sl.k_rem = sl.rank; S->slot[1][s] = sl; }
        s_prefix[s] = sl.prefix;
        s_grp[s] = sl.done ? -2 : -1;
    }
    sync();
    if (threadIdx.x == 0) {
        int G = 0;
        bool over = tl.ncls > DISCO_MAX_CLS || tl.ncls < 1;
        unsigned gp[DISCO_MAX_GRP] = {0u, 0u, 0u, 0u};
        for (int s = 0; s < ns; ++s) {
            int g = -1;
            if (s_grp[s] != -2) {
                const unsigned prefix = s_prefix[s];
#pragma unroll
                for (int k = 0; k < DISCO_MAX_GRP; ++k)
                    if (k < G && gp[k] == prefix) g = k;
                if (g < 0) {
                    if (G < DISCO_MAX_GRP) {
#pragma unroll
                        for (int k = 0; k < DISCO_MAX_GRP; ++k)
                            if (k == G) gp[k] = prefix;
                        g = G;
                    } else {
                        g = 0;         // too many distinct prefixes: the per-slot fallback does not use groups
                    }
                    G += 1;
                }
            }
            s_grp[s] = g;
        }
#pragma unroll
        for (int k = 0; k < DISCO_MAX_GRP; ++k)
            if (k < G) tl.grp_prefix[k] = gp[k];
        if (G > DISCO_MAX_GRP) over = true;
        if (over) tl.fallback = 1;
        tl.G = G;
        int w;
        if (over || tl.fallback) {
            w = fit_width(P * nq, DISCO_TL_HIST_WORDS);
        } else {
            const int g1 = G > 0 ? G : 1;
            w = fit_width((long)g1 * (tl.nwalk > 0 ? tl.nwalk : 1), DISCO_TL_HIST_WORDS);
            const int wg = fit_width((long)g1 * tl.ncls, DISCO_GHIST_WORDS);
            if (wg < w) w = wg;
        }
        if (w < 1) w = 1;
        if (w > tl.left) w = tl.left;
        if (G == 0) w = 0;                 // nothing left to select
        tl.width = w;
        tl.shift = tl.left - w;
    }
    sync();
    for (int s = threadIdx.x; s < ns; s += nt) tl.slot_grp[s] = s_grp[s];
}

// Distinct column sets of a workgroup's requests: an open-addressing hash table in LDS (CL_SLOTS slots, far more
// than the DISCO_MAX_CLS sets a class-mode selection can hold).  A lane looks its set up with one LDS read in the
// common case (lanes with the same set read the same slot); a new set is claimed with a compare-and-swap.
constexpr int CL_BLOCK = 1024;              // classification: 16 waves share one table
constexpr int CL_SLOTS = DISCO_CLS_SLOTS;

struct ClassTable {
    u64 slot[CL_SLOTS];            // 0 = free
    unsigned walk[CL_SLOTS];       // a member of the set needs a token walk
    u64 dense[DISCO_MAX_CLS];      // the sets, compacted (table_compact)
    unsigned long long dense_walk;
    unsigned wave_cnt[CL_BLOCK / 64];
    int overflow;
    unsigned plan_prefix[DISCO_MAX_SLOTS];     // scratch of the first plan (tbt_plan_next)
    int plan_grp[DISCO_MAX_SLOTS];
};

__device__ __forceinline__ void table_clear(ClassTable& T)
{
    for (int i = threadIdx.x; i < CL_SLOTS; i += CL_BLOCK) { T.slot[i] = 0ull; T.walk[i] = 0u; }
    if (threadIdx.x < DISCO_MAX_CLS) T.dense[threadIdx.x] = 0ull;
    if (threadIdx.x == 0) { T.dense_walk = 0ull; T.overflow = 0; }
}

__device__ __forceinline__ void table_insert(ClassTable& T, u64 m, bool walked)
{
    if (m == 0ull) return;
    unsigned h = (unsigned)((m * 0x9E3779B97F4A7C15ull) >> 56) & (CL_SLOTS - 1);
    volatile u64* vs = T.slot;
    for (int probe = 0; probe < CL_SLOTS; ++probe) {
        u64 cur = vs[h];
        if (cur == 0ull) cur = (u64)atomicCAS((unsigned long long*)&T.slot[h], 0ull, (unsigned long long)m);
        if (cur == 0ull || cur == m) {           // claimed now, or already there
            if (walked && ((volatile unsigned*)T.walk)[h] == 0u) ((volatile unsigned*)T.walk)[h] = 1u;
            return;
        }
        h = (h + 1) & (CL_SLOTS - 1);
    }
    T.overflow = 1;                              // (more than CL_SLOTS distinct sets)
}

// All threads: the occupied slots in slot order -> dense[0 .. count), dense_walk; more than DISCO_MAX_CLS -> overflow.
__device__ __forceinline__ int table_compact(ClassTable& T)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();
    const u64 v = threadIdx.x < CL_SLOTS ? T.slot[threadIdx.x] : 0ull;
    const u64 occ = __ballot(v != 0ull);
    if (lane == 0) T.wave_cnt[wave] = (unsigned)__popcll(occ);
    __syncthreads();
    int before = 0, total = 0;
    for (int w = 0; w < CL_SLOTS / 64; ++w) { const int c = (int)T.wave_cnt[w]; before += w < wave ? c : 0; total += c; }
    if (v != 0ull) {
        const int pos = before + __popcll(occ & ((1ull << lane) - 1ull));
        if (pos < DISCO_MAX_CLS) {
            T.dense[pos] = v;
            if (T.walk[threadIdx.x]) atomicOr(&T.dense_walk, 1ull << pos);
        }
    }
    if (threadIdx.x == 0 && total > DISCO_MAX_CLS) T.overflow = 1;
    __syncthreads();
    return total < DISCO_MAX_CLS ? total : DISCO_MAX_CLS;
}

// Column sets of every request -> classes.  Every workgroup collects its distinct sets in an LDS hash table
// and enters them (a few dozen) into a device-wide table of the same kind; the workgroup that takes the last
// ticket compacts that table, puts the sets in ascending order (so that the class numbers do not depend on
// timing), numbers the classes that need a token walk and plans the first histogram pass.  Also clears the length
// counts and the device-wide bins.  The device-wide table was zeroed when the selection started (select_init, in
// the launch that stages the policy table).
__global__ __launch_bounds__(CL_BLOCK) void k_tl_classify(TraceView tr, const disco_policy* __restrict__ pol, int P, int nq,
                                                     float tau, const TlSummary* __restrict__ summary,
                                                     const BufSummary* __restrict__ bufsum, SelState* S,
                                                     unsigned* ppcnt, unsigned* ghist, unsigned* dhist, unsigned* ticket)
{
    __shared__ disco_policy sp[DISCO_MAX_COLS];
    __shared__ ClassTable T;
    if ((int)threadIdx.x < P) sp[threadIdx.x] = pol[threadIdx.x];
    table_clear(T);
    for (i64 w = (i64)blockIdx.x * CL_BLOCK + threadIdx.x; w < (i64)DISCO_MAX_CLS * (DISCO_PP_NMAX + 1); w += (i64)gridDim.x * CL_BLOCK)
        ppcnt[w] = 0u;
    for (i64 w = (i64)blockIdx.x * CL_BLOCK + threadIdx.x; w < (i64)DISCO_GHIST_WORDS; w += (i64)gridDim.x * CL_BLOCK) ghist[w] = 0u;
    for (i64 w = (i64)blockIdx.x * CL_BLOCK + threadIdx.x; w < (i64)P * DISCO_DELAY_BINS; w += (i64)gridDim.x * CL_BLOCK) dhist[w] = 0u;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const i64 nround = (tr.n_req + CL_BLOCK - 1) / CL_BLOCK;
    for (i64 rnd = blockIdx.x; rnd < nround; rnd += gridDim.x) {
        const i64 i = rnd * CL_BLOCK + threadIdx.x;
        if (i >= tr.n_req) continue;
        const int l = tr.l[i], n = tr.n[i];
        const float s = tr.s[i];
        const float k = tr.k ? tr.k[i] : tr.k_s;
        u64 m[TL_KINDS];
        request_sets(sp, P, l, s, __fmaf_rn((float)l, k, tr.c), i, m);
        const TlSummary sm = summary[i];
        table_insert(T, m[TL_DEV], !timeline_is_analytic(TL_DEV, n, sm));
        table_insert(T, m[TL_SRV], !timeline_is_analytic(TL_SRV, n, sm));
        table_insert(T, m[TL_SRV_LAG], !timeline_is_analytic(TL_SRV_LAG, n, sm));
        if ((m[TL_SRV_BUF] | m[TL_DEV_BUF]) != 0ull) {
            const BufSummary bs = bufsum[i];
            table_insert(T, m[TL_SRV_BUF], !buf_timeline_is_analytic(TL_SRV_BUF, n, bs));
            table_insert(T, m[TL_DEV_BUF], !buf_timeline_is_analytic(TL_DEV_BUF, n, bs));
        }
    }
    {
        // this workgroup's distinct sets into the device-wide table (same probing; entries are never changed once
        // claimed, so a stale read can only cost an extra compare-and-swap)
        const int mine_n = table_compact(T);
        TlSel& g = S->tl;
        if ((int)threadIdx.x < mine_n) {
            const u64 m = T.dense[threadIdx.x];
            const bool walked = (T.dense_walk >> threadIdx.x) & 1ull;
            unsigned h = (unsigned)((m * 0x9E3779B97F4A7C15ull) >> 56) & (CL_SLOTS - 1);
            volatile u64* vs = g.gslot;
            bool placed = false;
            for (int probe = 0; probe < CL_SLOTS && !placed; ++probe) {
                u64 cur = vs[h];
                if (cur == 0ull) cur = (u64)atomicCAS((unsigned long long*)&g.gslot[h], 0ull, (unsigned long long)m);
                if (cur == 0ull || cur == m) {
                    if (walked && ((volatile unsigned*)g.gwalk)[h] == 0u) atomicOr(&g.gwalk[h], 1u);
                    placed = true;
                } else {
                    h = (h + 1) & (CL_SLOTS - 1);
                }
            }
            if (!placed) g.goverflow = 1;
        }
        if (threadIdx.x == 0 && T.overflow) g.goverflow = 1;
    }
    if (!take_last_ticket(ticket)) return;
    // last workgroup: the device-wide table (read where the atomics put it), compacted and put in order
    __syncthreads();
    table_clear(T);
    __syncthreads();
    if (threadIdx.x < CL_SLOTS) {
        T.slot[threadIdx.x] = (u64)atomicCAS((unsigned long long*)&S->tl.gslot[threadIdx.x], 0ull, 0ull);
        T.walk[threadIdx.x] = atomicOr(&S->tl.gwalk[threadIdx.x], 0u);
    }
    if (threadIdx.x == 0 && atomicOr((unsigned*)&S->tl.goverflow, 0u) != 0u) T.overflow = 1;
    const int total = table_compact(T);
    if (wave != 0) return;
    // ascending order: lane e holds a set, its rank is the number of smaller ones
    const u64 v = lane < total ? T.dense[lane] : ~0ull;
    int rank = 0;
    for (int j = 0; j < total; ++j) rank += bcast_u64(v, j) < v ? 1 : 0;
    TlSel& tl = S->tl;
    tl.cls_mask[lane < total ? rank : lane] = lane < total ? v : 0ull;
    // walk mask in the new numbering: bit `rank` of the lanes whose set is walked
    u64 wm = 0ull;
    for (int j = 0; j < total; ++j) {
        const int rj = bcast_i(rank, j);
        if ((T.dense_walk >> j) & 1ull) wm |= 1ull << rj;
    }
    {
        // rows of the walked classes in the workgroups' LDS histogram, in class order
        const bool wl = (wm >> lane) & 1ull;
        const int row = __popcll(wm & ((1ull << lane) - 1ull));
        tl.cls_slot[lane] = wl ? (signed char)row : (signed char)-1;
        u64 t = wm;                                          // class of row `lane`: the lane-th walked class
        for (int q = 0; q < lane && t != 0ull; ++q) t &= t - 1ull;
        tl.slot_cls[lane] = t != 0ull ? (unsigned char)(__ffsll((long long)t) - 1) : (unsigned char)0;
    }
    __builtin_amdgcn_wave_barrier();
    if (lane == 0) {
        tl.ncls = total > 0 ? total : 1;
        tl.walk_mask = wm;
        tl.nwalk = __popcll(wm);
        tl.error = 0;
        if (T.overflow) tl.fallback = 1;               // more than DISCO_MAX_CLS distinct sets: per-slot histograms
        // gaps sit just above the pacing interval (down to a few thousand ulps below it after rounding): try a
        // 21-bit window of keys first
        const unsigned tb = f2u(tau);
        tl.restart = 0;
        tl.nlist = 0u;
        tl.nlist_back = 0u;
        if (tb >= 8192u) { tl.key_lo = tb - 8192u; tl.window = 21; tl.left = 21; }
        else { tl.key_lo = 0u; tl.window = 0; tl.left = 31; }
        *ticket = 0u;
    }
    __builtin_amdgcn_wave_barrier();
    tbt_plan_next(S, P, nq, T.plan_prefix, T.plan_grp, true, false);
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

// Step 1 of a TBT pass (all threads of a workgroup, class c; beside the
// workgroups that walk tokens, hence atomic adds): add the analytic bins of
// the class's pure-pacing timelines to its device-wide rows.  ppcnt[c][t] timelines of class c have a token t, and the
// gap in front of it is the same number for all of them.
__device__ void analytic_class(SelState* S, unsigned* ghist, const unsigned* ppcnt, float tau, int c, unsigned* lds)
{
    const TlSel& tl = S->tl;
    const int width = tl.width, ncls = tl.ncls;
    const unsigned* row = ppcnt + (size_t)c * (DISCO_PP_NMAX + 1);
    if (row[0] == 0u) return;                             // no pure-pacing timeline in this class (uniform)
    const int Gused = tl.G < DISCO_MAX_GRP ? tl.G : DISCO_MAX_GRP;
    const unsigned dmask = (1u << width) - 1u;
    const int words = Gused << width;
    const int shift = tl.shift, up = tl.shift + width;
    const unsigned key_cap = tl.window ? (1u << tl.window) : 0xFFFFFFFFu;
    __syncthreads();
    for (int i = threadIdx.x; i < words; i += blockDim.x) lds[i] = 0u;
    __syncthreads();
    for (int t = 1 + (int)threadIdx.x; t < DISCO_PP_NMAX; t += blockDim.x) {
        const unsigned cnt = row[t];
        if (!cnt) continue;
        const unsigned key = tbt_key(f2u((float)t * tau - (float)(t - 1) * tau), tl.key_lo, key_cap);
        const unsigned hi = key >> up;                     // clamped keys match no prefix
        int g = -1;
        for (int k = 0; k < Gused; ++k) g = (hi == tl.grp_prefix[k] && g < 0) ? k : g;
        if (g >= 0) atomicAdd(&lds[((unsigned)g << width) | ((key >> shift) & dmask)], cnt);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < words; i += blockDim.x) {
        const unsigned v = lds[i];
        if (v) atomicAdd(&ghist[((size_t)((i >> width) * ncls + c) << width) | (i & dmask)], v);
    }
}

// Step 2 (all threads of a workgroup, (column, quantile) slot s): add up the
// class histograms of the classes that contain the slot's column (or take the
// slot's own histogram in the fallback), walk to the digit that holds the
// remaining rank, extend the prefix.
//   binsum: LDS scratch of binsum_cap words: the slot's bin counts are summed over its classes there with
//   coalesced reads of the class rows (a thread then scans consecutive bins from LDS); wider digits and the
//   fallback read the rows directly.
__device__ void select_slot(SelState* S, int nq, const unsigned* ghist, int s, u64* wsum /* LDS, 64 */, int* s_digit, u64* s_rem,
                            u64* binsum, int binsum_cap)
{
    const TlSel& tl = S->tl;
    const int width = tl.width, ncls = tl.ncls, fallback = tl.fallback;
    SelSlot sl = S->slot[1][s];
    const int g = tl.slot_grp[s];
    if (sl.done || g < 0) return;                         // uniform
    const int col = s / nq;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nbins = 1 << width;
    const int per = (nbins + (int)blockDim.x - 1) / (int)blockDim.x;      // consecutive bins per thread
    const int b0 = threadIdx.x * per;
    const bool staged = !fallback && nbins <= binsum_cap;
    if (staged) {
        // the classes that contain the column (the first wave lists them in wsum[0 .. nk), nk in *s_digit), then
        // every bin is the sum over their rows: all loads independent and coalesced
        __syncthreads();
        if (wave == 0) {
            const bool in = lane < ncls && ((tl.cls_mask[lane] >> col) & 1ull);
            const u64 inb = __ballot(in);
            if (in) wsum[__popcll(inb & ((1ull << lane) - 1ull))] = (u64)lane;
            if (lane == 0) *s_digit = __popcll(inb);
        }
        __syncthreads();
        const int nk = *s_digit;
        for (int b = threadIdx.x; b < nbins; b += (int)blockDim.x) {
            u64 c = 0;
#pragma unroll 4
            for (int j = 0; j < nk; ++j) c += ghist[((size_t)(g * ncls + (int)wsum[j]) << width) | b];
            binsum[b] = c;
        }
        __syncthreads();
    }
    auto bin_count = [&](int b) -> u64 {
        if (staged) return binsum[b];
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
    __syncthreads();
    if (lane == 63) wsum[wave] = incl;
    if (threadIdx.x == 0) *s_digit = -1;
    __syncthreads();
    u64 before = 0;
    for (int w = 0; w < wave; ++w) before += wsum[w];
    incl += before;
    const u64 k = (u64)sl.k_rem;
    if (incl >= k && incl - mine < k) {                   // at most one thread: the rank falls into its bins
        u64 rem = k - (incl - mine);
        int dsel = b0;
        for (int b = b0; b < b0 + per && b < nbins; ++b) {
            const u64 c = bin_count(b);
            dsel = b;
            if (rem <= c) break;
            rem -= c;
        }
        *s_digit = dsel;
        *s_rem = rem;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        int dsel = *s_digit;
        u64 rem = *s_rem;
        // window mode: a rank beyond the counted keys, or in the bottom bin (which also holds the keys below the
        // window), is not decided here -> start over on raw keys.  Raw keys: the rank is always found.
        if (tl.window && (dsel < 0 || (dsel == 0 && tl.left == tl.window))) S->tl.restart = 1;
        if (dsel < 0) { dsel = nbins - 1; rem = 1; }
        sl.k_rem = (i64)rem;
        sl.prefix = (sl.prefix << width) | (unsigned)dsel;
        S->slot[1][s] = sl;
    }
}

// Step 3 (one workgroup): clear the bins that were used and plan the next pass.
__device__ void plan_pass(SelState* S, int P, int nq, unsigned* ghist, unsigned* s_prefix, int* s_grp)
{
    TlSel& tl = S->tl;
    const int width = tl.width;
    const int Gused = tl.G < DISCO_MAX_GRP ? tl.G : DISCO_MAX_GRP;
    const int words = (tl.fallback ? P * nq : Gused * tl.ncls) << width;
    __syncthreads();
    for (int i = threadIdx.x; i < words; i += blockDim.x) ghist[i] = 0u;
    __syncthreads();
    const bool restart = tl.window && tl.restart;          // the window missed a rank: all slots start over on raw keys
    const bool more = restart || tl.left - width > 0;
    __syncthreads();                                       // (every thread has read the state thread 0 now changes)
    if (threadIdx.x == 0) {
        if (restart) { tl.window = 0; tl.key_lo = 0u; tl.restart = 0; tl.left = 31; }
        else if (more) tl.left -= width;
        else { tl.left = 0; tl.width = 0; tl.G = 0; }
    }
    __syncthreads();
    if (more) tbt_plan_next(S, P, nq, s_prefix, s_grp, false, restart);
}

// Workgroups of the launches below, by what they run.
struct PassGrid { unsigned analytic, fast, buf, general; };

__device__ __forceinline__ BufHistArgs buf_hist_args(const TimelineArgs& a)
{
    BufHistArgs h;
    h.h.tau = a.tau; h.h.kt = a.kt; h.h.P = a.P; h.h.pass = a.pass;
    h.h.S = a.S; h.h.ghist = a.ghist; h.h.desc = a.desc; h.h.list = a.list;
    h.bc = a.bc;
    h.buffer_flag = a.buffer_flag;
    return h;
}

static_assert(TH_BLOCK == 1024 && TBH_BLOCK == 1024 && TL_BLOCK == 1024, "the kinds of workgroup share launches");

// A regular pass, everything but the streaming kinds' walk (which has a kernel of its own, built for occupancy):
// the analytic bins of the classes, the buffer hand-off timelines, the per-slot histograms of a table whose
// column sets do not fit the class scheme.  One launch, workgroups by kind; the kinds a table does not use
// return at once.
__global__ __launch_bounds__(1024) void k_tbt_side(TraceView tr, i64 n_tok, int align, const disco_policy* __restrict__ pol,
                                                   TimelineArgs a, PassGrid g)
{
    __shared__ __align__(16) unsigned smem[DISCO_TL_HIST_WORDS];
    __shared__ TimelineLds lds;
    const TlSel& tl = a.S->tl;
    if (tl.width <= 0) return;                          // selection finished
    unsigned bid = blockIdx.x;
    if (bid < g.analytic) {
        if (!tl.fallback && (int)bid < tl.ncls) analytic_class(a.S, a.ghist, a.ppcnt, a.tau, (int)bid, smem);
        return;
    }
    bid -= g.analytic;
    if (bid < g.buf) {
        if (!tl.fallback && *a.buffer_flag != 0u) tl_hist_buf_body(smem, tr, n_tok, align, buf_hist_args(a), bid, g.buf);
        return;
    }
    bid -= g.buf;
    if (tl.fallback) timeline_body<true>(smem, lds, tr, n_tok, align, pol, a, bid, g.general);
}

// Workgroup = slot: the digit of the slot; the workgroup that finishes last clears the bins and plans the next pass.
__global__ __launch_bounds__(1024) void k_tbt_select(SelState* S, int P, int nq, unsigned* ghist, unsigned* ticket)
{
    __shared__ u64 wsum[DISCO_MAX_CLS];
    __shared__ int s_digit;
    __shared__ u64 s_rem;
    __shared__ u64 binsum[2048];
    if (S->tl.width <= 0) return;
    select_slot(S, nq, ghist, blockIdx.x, wsum, &s_digit, &s_rem, binsum, 2048);
    if (!take_last_ticket(ticket)) return;
    plan_pass(S, P, nq, ghist, reinterpret_cast<unsigned*>(binsum), reinterpret_cast<int*>(binsum + DISCO_MAX_SLOTS));
    if (threadIdx.x == 0) *ticket = 0u;
}

// A spare pass (after the passes that normally finish the selection: needed when the window was missed or the
// digits are narrow) in one launch: workgroups by kind walk the tokens, the one that finishes last adds the
// analytic bins, takes every slot's digit, clears the bins and plans the next pass.  One launch per pass matters
// more here than speed: normally all of them return at once.
__global__ __launch_bounds__(1024) void k_tbt_spare(TraceView tr, i64 n_tok, int align, const disco_policy* __restrict__ pol,
                                                    TimelineArgs a, PassGrid g)
{
    __shared__ __align__(16) unsigned smem[DISCO_TL_HIST_WORDS];
    __shared__ TimelineLds lds;
    __shared__ u64 wsum[DISCO_MAX_CLS];
    __shared__ int s_digit;
    __shared__ u64 s_rem;
    SelState* S = a.S;
    const TlSel& tl = S->tl;
    if (tl.width <= 0) return;                          // selection finished (the same answer in every workgroup)
    const unsigned bid = blockIdx.x;
    if (tl.fallback) {
        if (bid >= g.fast + g.buf) timeline_body<true>(smem, lds, tr, n_tok, align, pol, a, bid - g.fast - g.buf, g.general);
    } else if (bid < g.fast) {
        HistArgs h;
        h.tau = a.tau; h.kt = a.kt; h.P = a.P; h.pass = a.pass; h.S = a.S; h.ghist = a.ghist; h.desc = a.desc; h.list = a.list;
        tl_hist_fast_body(smem, tr, n_tok, align, h, bid, g.fast);
    } else if (bid < g.fast + g.buf) {
        if (*a.buffer_flag != 0u) tl_hist_buf_body(smem, tr, n_tok, align, buf_hist_args(a), bid - g.fast, g.buf);
    }
    if (!take_last_ticket(a.ticket)) return;
    if (!tl.fallback)
        for (int c = 0; c < tl.ncls; ++c) analytic_class(S, a.ghist, a.ppcnt, a.tau, c, smem);
    __syncthreads();
    for (int s = 0; s < a.P * a.nq; ++s) {
        select_slot(S, a.nq, a.ghist, s, wsum, &s_digit, &s_rem, reinterpret_cast<u64*>(smem), DISCO_TL_HIST_WORDS / 2);
        __syncthreads();
    }
    plan_pass(S, a.P, a.nq, a.ghist, smem, reinterpret_cast<int*>(smem + DISCO_MAX_SLOTS));
    if (threadIdx.x == 0) *a.ticket = 0u;
}

}  // namespace

void disco_launch_tl_classify(const TraceView& v, const disco_policy* pol, int P, int nq, float tau, const void* summary,
                              const void* bufsum, SelState* S, unsigned* ppcnt, unsigned* ghist, unsigned* dhist, unsigned* ticket,
                              hipStream_t stream)
{
    i64 b = (v.n_req + CL_BLOCK - 1) / CL_BLOCK;
    if (b < 1) b = 1;
    if (b > 256) b = 256;                          // (more workgroups cost more in the merge than they save in the scan)
    b /= disco_grid_divisor();
    if (b < 1) b = 1;
    hipLaunchKernelGGL(k_tl_classify, dim3((unsigned)b), dim3(CL_BLOCK), 0, stream, v, pol, P, nq, tau,
                       (const TlSummary*)summary, (const BufSummary*)bufsum, S, ppcnt, ghist, dhist, ticket);
}

void disco_launch_pp_suffix(SelState* S, unsigned* ppcnt, hipStream_t stream)
{
    hipLaunchKernelGGL(k_pp_suffix, dim3(DISCO_MAX_CLS), dim3(1024), 0, stream, S, ppcnt);
}

// One pass of the TBT selection over everything but the streaming kinds' walk in the regular passes (that walk:
// disco_launch_tl_hist_fast, before this), then the step to the next pass.
void disco_launch_tbt_pass(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a, hipStream_t stream)
{
    const int align = (int)(((uintptr_t)v.arr >> 2) & 3);
    const i64 per_wave = (v.n_req + 15) / 16;                    // workgroups if every wave took one request
    auto cap = [&](i64 c) { return (unsigned)(per_wave < 1 ? 1 : (per_wave > c ? c : per_wave)); };
    PassGrid g;
    if (a.pass < DISCO_TBT_REGULAR_PASS) {
        g.analytic = DISCO_MAX_CLS; g.fast = 0; g.buf = cap(512); g.general = cap(512);
        hipLaunchKernelGGL(k_tbt_side, dim3(g.analytic + g.buf + g.general), dim3(1024), 0, stream, v, n_tok, align, pol, a, g);
        hipLaunchKernelGGL(k_tbt_select, dim3((unsigned)(a.P * a.nq)), dim3(1024), 0, stream, a.S, a.P, a.nq, a.ghist, a.ticket);
    } else {
        // small grids: an empty launch is cheaper and a needed one merely slower
        g.analytic = 0; g.fast = cap(64); g.buf = cap(64); g.general = cap(128);
        hipLaunchKernelGGL(k_tbt_spare, dim3(g.fast + g.buf + g.general), dim3(1024), 0, stream, v, n_tok, align, pol, a, g);
    }
}
