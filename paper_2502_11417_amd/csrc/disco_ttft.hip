// TTFT order statistics (Sec. 5.1 metrics: median and tail TTFT per budget
// level): most-significant-digit-first radix selection over
// key = bits(TTFT) - min_bits, 8 bits per pass.
//
// Two kinds of histogram workgroups in one launch; which kind acts is decided on the device.
//
//   class kernel -- every column is a length-threshold column (Alg. 3).  With
//     the thresholds in ascending order t_0 <= ... <= t_{P-1} a request of
//     prompt length l runs device-only in the columns p >= ub and races in the
//     columns p < ub, ub = #{p : t_p <= l}; its TTFT is d in the former and
//     min(s, d) in the latter (the winner of a race does not depend on the
//     column).  So a request has at most two distinct TTFT values over the
//     whole table, each valid for a contiguous range of sorted columns:
//     lane = request, two histogram updates per request instead of one per
//     (request, column) pair.
//       pass 0: rows (device, ub) and (race, ub); column p's histogram is the
//         sum of the device rows ub <= p and the race rows ub > p.
//       second pass: the live (column, quantile) slots are grouped by their
//         first digit.  If all values that carry one of these digits fit the
//         candidate list, they are sorted into one bucket per digit (4-byte
//         entries: the undecided key bits and the column range of the value)
//         and every slot finishes its remaining digits from its bucket
//         (k_ttft_select, one workgroup per slot): no further pass over the
//         requests.
//       otherwise, histogram passes: one row per slot; a value goes to the
//         slots of its column range whose prefix equals the value's upper bits
//         (LDS hash of the distinct prefixes, 128-bit slot sets).
//   pair kernel -- any table: lane = column, every (request, column) pair is
//     evaluated and bumps the rows of its column.
//
// Without buckets, few values still match a slot's prefix after two passes
// (the second select adds up an upper bound): the third pass then collects
// them in a list -- key and which columns the value belongs to -- and every
// slot finishes its remaining digits from that list, instead of two more
// passes over the requests.  If that bound is too large as well (heavy ties)
// the histogram passes simply go on.
//
// A workgroup stores its LDS bins as one slice; k_ttft_reduce adds the slices
// (merging them with device-wide atomics would serialise on the few hundred
// cache lines of the bins) and k_ttft_select extends every slot's prefix.
#include <math.h>
#include <string.h>

#include <type_traits>

#include "disco_launch.h"
#include "disco_pair.h"
#include "disco_state.h"

namespace {

constexpr int TH_ROWS = 2 * DISCO_MAX_COLS + 2;         // class pass 0: (device, ub) 0..P and (race, ub) 0..P
constexpr int TH_PAD = 1;                               // skew: equal digits of different rows hit different banks
constexpr int TH_STRIDE = 256 + TH_PAD;
constexpr int TH_WORDS = TH_ROWS * TH_STRIDE;           // 131 KB of LDS bins
constexpr int TC_MAX_BLOCKS = 256;                      // class kernel: one workgroup per CU (its slices: TH_ROWS x 256 bins each)

struct PassDigit { int width, shift, up; unsigned dmask; };

// Candidate list of the finishing step: 2^21 entries of 8 bytes in the slice region.
constexpr unsigned TG_CAP = 1u << 21;
struct GEntry { unsigned key, tag; };           // tag: kind << 16 | u; kind 0: columns at sorted position >= u,
                                                // 1: columns at sorted position < u, 2: column u
__device__ __forceinline__ bool gather_on(const SelGlobal& g) { return g.plan.npass > 2 && g.gather_bound <= (u64)TG_CAP; }

// Entries are staged per wave in LDS (the histogram bins are idle in this pass): a wave appends to its own
// segment without atomics -- the count is wave-uniform -- and spills a full segment to the device-wide list; what is
// left at the end goes out with one device-wide atomic per workgroup (one per wave would queue up on the counter).
constexpr unsigned TG_SEG = TH_WORDS / 2 / DP_WAVES;            // entries per wave
struct WaveList { GEntry* seg; unsigned cnt; };

__device__ __forceinline__ void wl_copy(const WaveList& w, unsigned base, GEntry* __restrict__ list, SelGlobal* g)
{
    __builtin_amdgcn_wave_barrier();
    for (unsigned j = threadIdx.x & 63; j < w.cnt; j += 64) {
        if (base + j < TG_CAP) list[base + j] = w.seg[j];
        else g->gather_error = 1;                              // cannot happen while gather_bound holds
    }
    __builtin_amdgcn_wave_barrier();
}

// Called by all lanes of the wave.
__device__ __forceinline__ void wl_append(WaveList& w, bool match, unsigned key, unsigned tag, GEntry* __restrict__ list,
                                          SelGlobal* g)
{
    const int lane = threadIdx.x & 63;
    if (w.cnt + 64u > TG_SEG) {                                // wave-uniform
        unsigned base = 0u;
        if (lane == 0) base = atomicAdd(&g->n_list, w.cnt);
        base = (unsigned)__shfl((int)base, 0, 64);
        wl_copy(w, base, list, g);
        w.cnt = 0u;
    }
    const u64 m = __ballot(match);
    if (match) w.seg[w.cnt + (unsigned)__popcll(m & ((1ull << lane) - 1ull))] = GEntry{key, tag};
    w.cnt += (unsigned)__popcll(m);
}

// Called by all threads of the workgroup.
__device__ __forceinline__ void wl_finish(const WaveList& w, GEntry* __restrict__ list, SelGlobal* g)
{
    __shared__ unsigned woff[DP_WAVES + 1];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0) woff[wave] = w.cnt;
    __syncthreads();
    if (threadIdx.x == 0) {
        unsigned total = 0u;
        for (int k = 0; k < DP_WAVES; ++k) { const unsigned c = woff[k]; woff[k] = total; total += c; }
        woff[DP_WAVES] = total ? atomicAdd(&g->n_list, total) : 0u;
    }
    __syncthreads();
    wl_copy(w, woff[DP_WAVES] + woff[wave], list, g);
}

__device__ __forceinline__ PassDigit pass_digit(const SelGlobal& g, int pass)
{
    PassDigit d;
    d.width = pass < g.plan.npass ? g.plan.width[pass] : 0;
    d.shift = pass < g.plan.npass ? g.plan.shift[pass] : 0;
    d.up = d.shift + d.width;                           // 32 only when the prefix is empty
    d.dmask = (1u << d.width) - 1u;
    return d;
}

__device__ __forceinline__ void store_slice(const unsigned* hist, int rows, int width, unsigned* __restrict__ slices, int bid)
{
    unsigned* mine = slices + (size_t)bid * ((size_t)rows << width);
    const int dmask = (1 << width) - 1;
    for (int i = threadIdx.x; i < rows << width; i += DP_BLOCK) mine[i] = hist[(i >> width) * TH_STRIDE + (i & dmask)];
}

// ------------------------------------------------------------ pair kernel --

// Same traversal as the fused dispatch pass; every pair whose key matches the
// prefix of a (column, quantile) slot bumps that slot's bin.  Pass 0: one row
// per column (all quantiles share it).
template <int G>
__device__ __forceinline__ void pair_body(const TraceView& tr, const disco_policy* __restrict__ pol, int P, int nq, int pass,
                                          SelState* S, unsigned* __restrict__ slices, unsigned* hist, Staged* stage,
                                          int bid, int nblk, bool gather)
{
    const SelGlobal g = S->g[0];
    const PassDigit dg = pass_digit(g, pass);
    if (dg.width <= 0) return;
    GEntry* list = reinterpret_cast<GEntry*>(slices);
    WaveList wl{reinterpret_cast<GEntry*>(hist) + (threadIdx.x >> 6) * TG_SEG, 0u};
    const int width = dg.width, shift = dg.shift, up = dg.up;
    const unsigned dmask = dg.dmask;
    const int nslot = (pass == 0) ? P : P * nq;
    for (int i = threadIdx.x; i < nslot * TH_STRIDE; i += DP_BLOCK) hist[i] = 0u;
    __syncthreads();
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & (G - 1), sub = lane / G;
    const bool colv = col < P;
    const disco_policy p = pol[colv ? col : 0];
    const StochRuns runs = stoch_runs(p, colv, lane);
    unsigned prefix[DISCO_MAX_Q];
    bool live[DISCO_MAX_Q];
    bool any_live = false;
#pragma unroll
    for (int qi = 0; qi < DISCO_MAX_Q; ++qi) {
        const bool on = colv && qi < nq;
        const SelSlot sl = S->slot[0][on ? col * nq + qi : 0];
        prefix[qi] = sl.prefix;
        live[qi] = on && !sl.done;
        any_live = any_live || live[qi];
    }
    Staged* st = stage + wave * 64;
    const i64 nbatch = (tr.n_req + 63) >> 6;
    // the pair evaluation is specialised on the kind of table (all Alg. 3, all Alg. 2, mixed)
    auto run = [&](auto mode_c) {
        constexpr int MODE = decltype(mode_c)::value;
        for (i64 b = (i64)bid * DP_WAVES + wave; b < nbatch; b += (i64)nblk * DP_WAVES) {
            const i64 i = b * 64 + lane;
            const bool v = i < tr.n_req;
            const int lv = v ? tr.l[i] : 0;
            const float sv = v ? tr.s[i] : 0.0f;
            const float kv = tr.k ? (v ? tr.k[i] : 0.0f) : tr.k_s;
            const float dv = __fmaf_rn((float)lv, kv, tr.c);
            st[lane] = Staged{lv, sv, 0, dv};
            const int cnt = (int)((tr.n_req - b * 64 < 64) ? (tr.n_req - b * 64) : 64);
            const bool shared = MODE == 2 && runs.on;       // stochastic columns: one draw per request and run
            float su[STOCH_SHARE] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
            if (shared) stoch_draw(runs, i, su);
            __builtin_amdgcn_wave_barrier();
#pragma unroll 4
            for (int it = 0; it < G; ++it) {
                const int src = sub * G + it;
                const Staged r = st[src];
                const float u = shared ? stoch_fetch<G == 64>(runs, su, src) : 0.0f;
                const PairResult e = pair_eval<MODE>(p, r.l, r.s, r.d, b * 64 + src, shared, u);
                if (gather) {                            // collect the pairs that still match a slot of their column
                    const unsigned key = f2u(e.ttft) - g.minb;
                    const unsigned hi = key >> up;
                    bool match = false;
#pragma unroll
                    for (int qi = 0; qi < DISCO_MAX_Q; ++qi) match = match || (live[qi] && hi == prefix[qi]);
                    wl_append(wl, match && src < cnt, key, 0x20000u | (unsigned)col, list, &S->g[0]);
                } else if (src < cnt) {
                    const unsigned key = f2u(e.ttft) - g.minb;
                    const unsigned dgt = (key >> shift) & dmask;
                    const unsigned hi = (up >= 32) ? 0u : (key >> up);
                    if (pass == 0) {
                        if (any_live) atomicAdd(&hist[col * TH_STRIDE + dgt], 1u);
                    } else {
#pragma unroll
                        for (int qi = 0; qi < DISCO_MAX_Q; ++qi)
                            if (live[qi] && hi == prefix[qi]) atomicAdd(&hist[(col * nq + qi) * TH_STRIDE + dgt], 1u);
                    }
                }
            }
            __builtin_amdgcn_wave_barrier();
        }
    };
    const int mode = table_mode(p, colv);
    if (mode == 0) run(std::integral_constant<int, 0>{});
    else if (mode == 1) run(std::integral_constant<int, 1>{});
    else run(std::integral_constant<int, 2>{});
    if (gather) { wl_finish(wl, list, &S->g[0]); return; }
    __syncthreads();
    store_slice(hist, nslot, width, slices, bid);
}

// ----------------------------------------------------------- class kernel --

// LDS tables of the class kernel's later passes.
struct ClsTables {
    int sorted[DISCO_MAX_COLS];                  // thresholds in ascending order (unused tail: INT_MAX)
    u64 dslots[DISCO_MAX_COLS + 1][2];           // slots of the columns p >= ub, as a 128-bit set
    u64 dmask[DISCO_MAX_SLOTS][2];               // live slots with the same prefix, kept at the first of them
    u64 htab[2 * DISCO_MAX_SLOTS];               // open-addressing hash: prefix -> first slot holding it (0: empty)
    unsigned sprefix[DISCO_MAX_SLOTS];
    int slive[DISCO_MAX_SLOTS];
    int first_of[DISCO_MAX_SLOTS];               // smallest live slot with the same prefix
    unsigned bbase[DISCO_MAX_SLOTS];             // scatter pass: first entry of a bucket in the list and the entry
    unsigned bend[DISCO_MAX_SLOTS];              // behind its last; entries of this workgroup for it in this round,
    unsigned bcnt[DISCO_MAX_SLOTS];              // and where they go
    unsigned bat[DISCO_MAX_SLOTS];
    int scatter;
    unsigned char col_of_pos[DISCO_MAX_COLS];
};

__device__ __forceinline__ unsigned prefix_hash(unsigned prefix) { return (prefix * 0x9E3779B1u) >> 24; }

// First slot holding `prefix`, -1 if no live slot does.  At most half of the table is occupied.
__device__ __forceinline__ int prefix_lookup(const ClsTables& T, unsigned prefix)
{
    unsigned h = prefix_hash(prefix);
    for (;;) {
        const u64 e = T.htab[h];
        if (e == 0ull) return -1;
        if ((unsigned)(e >> 8) == prefix) return (int)(e & 0xFFull);
        h = (h + 1u) & (2 * DISCO_MAX_SLOTS - 1);
    }
}

// ub = #{p : t_p <= l}: binary search over the 64 padded thresholds (the first pass leaves it in the request's
// workspace byte for the later ones when the caller's workspace has room).
__device__ __forceinline__ int request_ub(const ClsTables& T, int P, int l)
{
    int ub = 0;
#pragma unroll
    for (int step = 64; step >= 1; step >>= 1)
        if (ub + step <= DISCO_MAX_COLS && T.sorted[ub + step - 1] <= l) ub += step;
    return ub < P ? ub : P;
}

// Requests of a workgroup are taken four strides at a time: the loads of all four are issued before the first is used.
constexpr int TC_UNROLL = 4;

__device__ __forceinline__ void cls_body(const TraceView& tr, int P, int nq, int pass, SelState* S,
                                         unsigned* __restrict__ slices, unsigned* hist, ClsTables& T, int bid, int nblk,
                                         bool gather, unsigned char* __restrict__ ubytes, const unsigned* __restrict__ rowsum)
{
    const SelGlobal g = S->g[0];
    const PassDigit dg = pass_digit(g, pass);
    if (dg.width <= 0) return;
    const int width = dg.width, shift = dg.shift, up = dg.up;
    const unsigned dmask = dg.dmask;
    const int nslot = P * nq;
    const int rows = (pass == 0) ? 2 * (P + 1) : nslot;
    const int t = threadIdx.x;
    const bool may_scatter = pass == 1 && g.plan.npass >= 2;
    // the slot records travel from device memory while the bins are cleared
    SelSlot sl;
    const bool in = pass > 0 && t < nslot;
    if (in) sl = S->slot[0][t];
    if (!gather && !may_scatter)
        for (int i = t; i < rows * TH_STRIDE; i += DP_BLOCK) hist[i] = 0u;
    if (t < DISCO_MAX_COLS) { T.sorted[t] = t < P ? S->tc.sorted_lth[t] : 0x7FFFFFFF; T.col_of_pos[t] = S->tc.col_of_pos[t]; }
    if (pass > 0) {
        // tables of this pass, built without atomics
        if (t < DISCO_MAX_SLOTS) {
            T.slive[t] = in && !sl.done;
            T.sprefix[t] = (in && !sl.done) ? sl.prefix : 0xFFFFFFFFu;     // keys have 31 bits: never a prefix
        }
        if (t < 2 * DISCO_MAX_SLOTS) T.htab[t] = 0ull;
        __syncthreads();
        if (t < DISCO_MAX_SLOTS) {
            // live slots with the same prefix: every thread walks the 128 prefixes (broadcast reads)
            const unsigned mine = T.sprefix[t];
            const bool live = mine != 0xFFFFFFFFu;
            u64 m0 = 0ull, m1 = 0ull;
#pragma unroll 8
            for (int z = 0; z < 64; ++z) {
                m0 |= (T.sprefix[z] == mine) ? (1ull << z) : 0ull;
                m1 |= (T.sprefix[64 + z] == mine) ? (1ull << z) : 0ull;
            }
            if (!live) { m0 = 0ull; m1 = 0ull; }
            T.dmask[t][0] = m0; T.dmask[t][1] = m1;
            const int f = m0 ? __ffsll((long long)m0) - 1 : (m1 ? 64 + __ffsll((long long)m1) - 1 : t);
            T.first_of[t] = f;
            if (live && f == t) {                       // one hash entry per distinct prefix
                const u64 entry = ((u64)mine << 8) | (u64)t | (1ull << 63);
                unsigned h = prefix_hash(mine);
                while (atomicCAS((unsigned long long*)&T.htab[h], 0ull, (unsigned long long)entry) != 0ull)
                    h = (h + 1u) & (2 * DISCO_MAX_SLOTS - 1);
            }
        } else if (t < DISCO_MAX_SLOTS + 64) {
            // slots of the sorted columns p >= ub: suffix OR over the wave (lane = sorted position)
            const int p = t - DISCO_MAX_SLOTS;
            u64 b0 = 0ull, b1 = 0ull;
            if (p < P) {
                const int c = T.col_of_pos[p];
                for (int qi = 0; qi < nq; ++qi) {
                    const int sidx = c * nq + qi;
                    if (sidx < 64) b0 |= 1ull << sidx; else b1 |= 1ull << (sidx - 64);
                }
            }
#pragma unroll
            for (int d = 1; d < 64; d <<= 1) {
                const u64 o0 = shfl_down_u64(b0, d), o1 = shfl_down_u64(b1, d);
                if (p + d < 64) { b0 |= o0; b1 |= o1; }
            }
            T.dslots[p][0] = b0; T.dslots[p][1] = b1;
            if (p == 0) { T.dslots[DISCO_MAX_COLS][0] = 0ull; T.dslots[DISCO_MAX_COLS][1] = 0ull; }
        }
    }
    __syncthreads();
    bool scatter = false;
    if (may_scatter) {
        // Second pass: the live slots are grouped by their first digit (tables above: first_of names the group).
        // A group's bucket can take every value of the first pass with that digit (all rows of the row sums); if
        // the buckets of all groups fit the list, the values are sorted into them and the slots finish from there,
        // else this is a histogram pass.  Every workgroup plans the same buckets; the first one leaves the plan
        // to the select kernel.
        unsigned* psum = hist;                              // the bins are idle
        const int w0 = g.plan.width[0];
        {
            const int f = t & (DISCO_MAX_SLOTS - 1), part = t / DISCO_MAX_SLOTS;
            unsigned a = 0u;
            if (T.slive[f] && T.first_of[f] == f)
                for (int row = part; row < 2 * (P + 1); row += DP_BLOCK / DISCO_MAX_SLOTS)
                    a += rowsum[((size_t)row << w0) + T.sprefix[f]];
            psum[t] = a;
        }
        __syncthreads();
        if (t < DISCO_MAX_SLOTS) {
            unsigned a = 0u;
            for (int part = 0; part < DP_BLOCK / DISCO_MAX_SLOTS; ++part) a += psum[part * DISCO_MAX_SLOTS + t];
            T.bcnt[t] = a;
        }
        __syncthreads();
        if (t < DISCO_MAX_SLOTS) {
            u64 at = 0;
            for (int z = 0; z < t; ++z) at += ((u64)T.bcnt[z] + 3ull) & ~3ull;      // buckets start at multiples of four entries
            const u64 end = at + T.bcnt[t];
            T.bbase[t] = (unsigned)(at < TG_CAP ? at : TG_CAP);
            T.bend[t] = (unsigned)(end < TG_CAP ? end : TG_CAP);
            if (t == DISCO_MAX_SLOTS - 1) T.scatter = end <= (u64)TG_CAP;
        }
        __syncthreads();
        scatter = T.scatter != 0;
        if (bid == 0 && t < DISCO_MAX_SLOTS) {
            S->tb.base[t] = T.bbase[t]; S->tb.cap[t] = T.bend[t] - T.bbase[t];
            S->tb.of_slot[t] = T.slive[t] ? T.first_of[t] : -1;
            if (t == 0) S->tb.on = scatter ? 1 : 0;
        }
        if (!scatter) {
            __syncthreads();                                // psum has been read
            for (int i = t; i < rows * TH_STRIDE; i += DP_BLOCK) hist[i] = 0u;
            __syncthreads();
        }
    }
    const bool cached = ubytes != nullptr && pass > 0;
    const i64 stride = (i64)nblk * DP_BLOCK;
    if (scatter) {
        // same matching as a histogram pass, but the value goes to the bucket of its digit: positions inside the
        // workgroup's share of a bucket from an LDS counter, the share itself from one device-wide atomic per
        // bucket, workgroup and round of TC_UNROLL strides
        // (an entry: the key's undecided bits below the first digit, the tag's position in bits 24..30, its kind in bit 31)
        unsigned* list = slices;
        const unsigned lowmask = (1u << up) - 1u;
        for (i64 base = (i64)bid * DP_BLOCK; base < tr.n_req; base += TC_UNROLL * stride) {
            if (t < DISCO_MAX_SLOTS) T.bcnt[t] = 0u;
            bool v[TC_UNROLL];
            int l[TC_UNROLL], ubc[TC_UNROLL];
            float sv[TC_UNROLL], kv[TC_UNROLL];
#pragma unroll
            for (int q = 0; q < TC_UNROLL; ++q) {
                const i64 i = base + q * stride + t;
                v[q] = i < tr.n_req;
                l[q] = v[q] ? tr.l[i] : 0;
                sv[q] = v[q] ? tr.s[i] : 0.0f;
                kv[q] = tr.k ? (v[q] ? tr.k[i] : 0.0f) : tr.k_s;
                ubc[q] = (cached && v[q]) ? (int)ubytes[i] : 0;
            }
            __syncthreads();
            unsigned eent[2 * TC_UNROLL], epos[2 * TC_UNROLL];
            int ebkt[2 * TC_UNROLL];
#pragma unroll
            for (int q = 0; q < TC_UNROLL; ++q) {
                const float s = sv[q];
                const float d = __fmaf_rn((float)l[q], kv[q], tr.c);
                const int ub = v[q] ? (cached ? ubc[q] : request_ub(T, P, l[q])) : 0;
                const bool dev_wins = d < s;
                const int ub0 = dev_wins ? 0 : ub;
                const bool two = !dev_wins && ub > 0;
#pragma unroll
                for (int which = 0; which < 2; ++which) {
                    const int e = 2 * q + which;
                    const unsigned key = (which ? f2u(s) : f2u(d)) - g.minb;
                    const int u = which ? ub : ub0;
                    int f = -1;
                    if (v[q] && (which ? two : ub0 < P)) {
                        f = prefix_lookup(T, key >> up);
                        if (f >= 0) {
                            u64 m0 = T.dmask[f][0], m1 = T.dmask[f][1];
                            if (which) { m0 &= ~T.dslots[u][0]; m1 &= ~T.dslots[u][1]; }
                            else { m0 &= T.dslots[u][0]; m1 &= T.dslots[u][1]; }
                            if ((m0 | m1) == 0ull) f = -1;
                        }
                    }
                    eent[e] = (key & lowmask) | ((unsigned)u << 24) | ((unsigned)which << 31); ebkt[e] = f;
                    epos[e] = f >= 0 ? atomicAdd(&T.bcnt[f], 1u) : 0u;
                }
            }
            __syncthreads();
            if (t < DISCO_MAX_SLOTS && T.bcnt[t]) T.bat[t] = T.bbase[t] + atomicAdd(&S->tb.fill[t], T.bcnt[t]);
            __syncthreads();
#pragma unroll
            for (int e = 0; e < 2 * TC_UNROLL; ++e) {
                if (ebkt[e] < 0) continue;
                const unsigned at = T.bat[ebkt[e]] + epos[e];
                if (at < T.bend[ebkt[e]]) list[at] = eent[e];
                else S->g[0].gather_error = 1;                  // a bucket takes every value with its digit: never expected
            }
            __syncthreads();
        }
        return;
    }
    if (gather) {
        // same matching as a histogram pass, but the value is appended to the candidate list (all lanes of a
        // wave stay together: the append is a wave operation)
        GEntry* list = reinterpret_cast<GEntry*>(slices);
        WaveList wl{reinterpret_cast<GEntry*>(hist) + (threadIdx.x >> 6) * TG_SEG, 0u};
        for (i64 base = (i64)bid * DP_BLOCK; base < tr.n_req; base += TC_UNROLL * stride) {
            bool v[TC_UNROLL];
            int l[TC_UNROLL], ubc[TC_UNROLL];
            float sv[TC_UNROLL], kv[TC_UNROLL];
#pragma unroll
            for (int q = 0; q < TC_UNROLL; ++q) {
                const i64 i = base + q * stride + t;
                v[q] = i < tr.n_req;
                l[q] = v[q] ? tr.l[i] : 0;
                sv[q] = v[q] ? tr.s[i] : 0.0f;
                kv[q] = tr.k ? (v[q] ? tr.k[i] : 0.0f) : tr.k_s;
                ubc[q] = (cached && v[q]) ? (int)ubytes[i] : 0;
            }
#pragma unroll
            for (int q = 0; q < TC_UNROLL; ++q) {
                if (base + q * stride >= tr.n_req) break;           // the same for the whole workgroup
                const float s = sv[q];
                const float d = __fmaf_rn((float)l[q], kv[q], tr.c);
                const int ub = v[q] ? (cached ? ubc[q] : request_ub(T, P, l[q])) : 0;
                const bool dev_wins = d < s;
                const int ub0 = dev_wins ? 0 : ub;
                const bool two = !dev_wins && ub > 0;
#pragma unroll
                for (int which = 0; which < 2; ++which) {
                    const unsigned key = (which ? f2u(s) : f2u(d)) - g.minb;
                    const int u = which ? ub : ub0;
                    bool match = v[q] && (which ? two : ub0 < P);
                    if (match) {
                        const int f = prefix_lookup(T, key >> up);
                        match = f >= 0;
                        if (match) {
                            u64 m0 = T.dmask[f][0], m1 = T.dmask[f][1];
                            if (which) { m0 &= ~T.dslots[u][0]; m1 &= ~T.dslots[u][1]; }
                            else { m0 &= T.dslots[u][0]; m1 &= T.dslots[u][1]; }
                            match = (m0 | m1) != 0ull;
                        }
                    }
                    wl_append(wl, match, key, ((unsigned)which << 16) | (unsigned)u, list, &S->g[0]);
                }
            }
        }
        wl_finish(wl, list, &S->g[0]);
        return;
    }
    for (i64 i0 = (i64)bid * DP_BLOCK + t; i0 < tr.n_req; i0 += TC_UNROLL * stride) {
        bool v[TC_UNROLL];
        int l[TC_UNROLL], ubc[TC_UNROLL];
        float sv[TC_UNROLL], kv[TC_UNROLL];
#pragma unroll
        for (int q = 0; q < TC_UNROLL; ++q) {
            const i64 i = i0 + q * stride;
            v[q] = i < tr.n_req;
            l[q] = v[q] ? tr.l[i] : 0;
            sv[q] = v[q] ? tr.s[i] : 0.0f;
            kv[q] = tr.k ? (v[q] ? tr.k[i] : 0.0f) : tr.k_s;
            ubc[q] = (cached && v[q]) ? (int)ubytes[i] : 0;
        }
#pragma unroll
        for (int q = 0; q < TC_UNROLL; ++q) {
            if (!v[q]) continue;
            const i64 i = i0 + q * stride;
            const float s = sv[q];
            const float d = __fmaf_rn((float)l[q], kv[q], tr.c);
            const int ub = cached ? ubc[q] : request_ub(T, P, l[q]);
            if (pass == 0 && ubytes) ubytes[i] = (unsigned char)ub;
            const bool dev_wins = d < s;                    // ties go to the server
            // value 0: d for the columns p >= ub (for every column if the device also wins the races);
            // value 1: s for the columns p < ub
            const int ub0 = dev_wins ? 0 : ub;
            const bool two = !dev_wins && ub > 0;
            const unsigned key0 = f2u(d) - g.minb, key1 = f2u(s) - g.minb;
            if (pass == 0) {
                if (ub0 < P) atomicAdd(&hist[ub0 * TH_STRIDE + ((key0 >> shift) & dmask)], 1u);
                if (two) atomicAdd(&hist[(P + 1 + ub) * TH_STRIDE + ((key1 >> shift) & dmask)], 1u);
            } else {
#pragma unroll
                for (int which = 0; which < 2; ++which) {
                    if (which == 1 && !two) continue;
                    if (which == 0 && ub0 >= P) continue;
                    const unsigned key = which ? key1 : key0;
                    const int f = prefix_lookup(T, key >> up);          // up < 32 after the first pass
                    if (f < 0) continue;
                    const int u = which ? ub : ub0;
                    u64 m0 = T.dmask[f][0], m1 = T.dmask[f][1];
                    if (which) { m0 &= ~T.dslots[u][0]; m1 &= ~T.dslots[u][1]; }
                    else { m0 &= T.dslots[u][0]; m1 &= T.dslots[u][1]; }
                    const unsigned dgt = (key >> shift) & dmask;
                    while (m0) { const int sidx = __ffsll((long long)m0) - 1; m0 &= m0 - 1; atomicAdd(&hist[sidx * TH_STRIDE + dgt], 1u); }
                    while (m1) { const int sidx = 64 + __ffsll((long long)m1) - 1; m1 &= m1 - 1; atomicAdd(&hist[sidx * TH_STRIDE + dgt], 1u); }
                }
            }
        }
    }
    __syncthreads();
    store_slice(hist, rows, width, slices, bid);
}

// One launch for both histogram kernels: workgroups [0, ncls_blocks) are the class kernel, the rest the pair
// kernel; the ones whose kind does not apply to the table return at once.
template <int G>
__global__ __launch_bounds__(DP_BLOCK) void k_ttft_hist(TraceView tr, const disco_policy* __restrict__ pol, int P, int nq,
                                                        int pass, SelState* S, unsigned* __restrict__ slices,
                                                        int ncls_blocks, unsigned char* __restrict__ ubytes,
                                                        const unsigned* __restrict__ rowsum)
{
    __shared__ unsigned hist[TH_WORDS];
    __shared__ __align__(16) Staged stage[DP_BLOCK];
    __shared__ ClsTables T;
    const bool cls_block = (int)blockIdx.x < ncls_blocks;
    if (cls_block != (S->tc.on != 0)) return;
    if (pass >= 2 && S->tb.on) return;                    // the buckets finished the selection
    const bool gather = pass >= 2 && gather_on(S->g[0]);
    if (gather && pass > 2) return;                       // the list finished the selection
    if (cls_block) cls_body(tr, P, nq, pass, S, slices, hist, T, blockIdx.x, ncls_blocks, gather, ubytes, rowsum);
    else pair_body<G>(tr, pol, P, nq, pass, S, slices, hist, stage, (int)blockIdx.x - ncls_blocks, (int)gridDim.x - ncls_blocks,
                      gather);
}

// ------------------------------------------------------ reduce and select --

// Adds the workgroup slices of one histogram row (workgroup = row; thread =
// (bin, quarter of the slices)).
__global__ __launch_bounds__(1024) void k_ttft_reduce(const SelState* S, int pass, int rows_pair, int rows_cls, int nsl_pair,
                                                      int nsl_cls, const unsigned* __restrict__ slices, unsigned* rowsum)
{
    __shared__ unsigned part[1024];
    const PassDigit dg = pass_digit(S->g[0], pass);
    if (dg.width <= 0) return;
    const int cls = S->tc.on;
    const int rows = cls ? rows_cls : rows_pair, nsl = cls ? nsl_cls : nsl_pair;
    const int row = blockIdx.x;
    if (row >= rows) return;
    const int bin = threadIdx.x & 255, q = threadIdx.x >> 8;
    unsigned a0 = 0, a1 = 0, a2 = 0, a3 = 0;
    if (bin < (1 << dg.width)) {
        const size_t step = (size_t)rows << dg.width;
        const unsigned* src = slices + ((size_t)row << dg.width) + bin;
        int b = q;
        for (; b + 12 < nsl; b += 16) {
            a0 += src[(size_t)b * step]; a1 += src[(size_t)(b + 4) * step];
            a2 += src[(size_t)(b + 8) * step]; a3 += src[(size_t)(b + 12) * step];
        }
        for (; b < nsl; b += 4) a0 += src[(size_t)b * step];
    }
    part[threadIdx.x] = (a0 + a1) + (a2 + a3);
    __syncthreads();
    if (q == 0 && bin < (1 << dg.width))
        rowsum[((size_t)row << dg.width) + bin] = part[bin] + part[256 + bin] + part[512 + bin] + part[768 + bin];
}

// The slot's remaining R digits from n candidates (workgroup = slot): histograms of up to 12 bits at a time (one
// scan when 12 bits or fewer are left) over the entries that carry the slot's prefix and belong to its column.
// PACKED = false: the list of the third pass, 8-byte entries {key, tag}.  PACKED = true: the bucket of the slot's
// first digit, 4-byte entries: the key's R undecided bits, above them (bits 24..30) the position u and (bit 31)
// the kind of the tag.  `list` is 16-byte aligned and readable up to 8 entries past n.
template <bool PACKED>
__device__ void finish_from_list(SelState* S, int s, int col, SelSlot sl, const void* __restrict__ list_, unsigned n, int R)
{
    constexpr int FW = 12, FB = 1 << FW;
    __shared__ unsigned fh[FB];
    __shared__ unsigned chosen;
    __shared__ u64 k_next, fsum[16];
    const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
    const unsigned pos = S->tc.on ? S->tc.pos_of_col[col] : 0u;
    const int R0 = R;
    const unsigned low0 = R0 < 32 ? (1u << R0) - 1u : 0xFFFFFFFFu;
    unsigned prefix = sl.prefix;
    u64 k = (u64)sl.k_rem;
    while (R > 0) {
        const int w = R < FW ? R : FW, sh = R - w;
        const unsigned dm = (1u << w) - 1u;
        const unsigned want = PACKED ? (prefix & ((1u << (R0 - R)) - 1u)) : prefix;     // PACKED: the digits found in the bucket
        for (int i = t; i < FB; i += blockDim.x) fh[i] = 0u;
        if (t == 0) chosen = 0xFFFFFFFFu;
        __syncthreads();
        auto take = [&](unsigned key, unsigned kind, unsigned u, bool valid) {
            const bool mine = kind == 0u ? pos >= u : (kind == 1u ? pos < u : (unsigned)col == u);
            if (valid && mine && (key >> R) == want) atomicAdd(&fh[(key >> sh) & dm], 1u);
        };
        if (PACKED) {
            const unsigned* list = static_cast<const unsigned*>(list_);
            for (unsigned e0 = 8u * t; e0 < n; e0 += 8u * blockDim.x) {
                const uint4 a = *reinterpret_cast<const uint4*>(&list[e0]);
                const uint4 b = *reinterpret_cast<const uint4*>(&list[e0 + 4]);
                const unsigned e[8] = {a.x, a.y, a.z, a.w, b.x, b.y, b.z, b.w};
#pragma unroll
                for (int q = 0; q < 8; ++q) take(e[q] & low0, e[q] >> 31, (e[q] >> 24) & 0x7Fu, e0 + q < n);
            }
        } else {
            const GEntry* list = static_cast<const GEntry*>(list_);
            for (unsigned e0 = 4u * t; e0 < n; e0 += 4u * blockDim.x) {
                const uint4 a = *reinterpret_cast<const uint4*>(&list[e0]);
                const uint4 b = *reinterpret_cast<const uint4*>(&list[e0 + 2]);
                const unsigned key[4] = {a.x, a.z, b.x, b.z}, tag[4] = {a.y, a.w, b.y, b.w};
#pragma unroll
                for (int q = 0; q < 4; ++q) take(key[q], tag[q] >> 16, tag[q] & 0xFFFFu, e0 + q < n);
            }
        }
        __syncthreads();
        // bins 4t .. 4t+3 per thread, inclusive prefix over the workgroup
        unsigned c[4];
        u64 mine = 0;
#pragma unroll
        for (int q = 0; q < 4; ++q) { c[q] = fh[4 * t + q]; mine += c[q]; }
        u64 incl = mine;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const unsigned lo = (unsigned)__shfl_up((int)(unsigned)incl, d, 64);
            const unsigned hi = (unsigned)__shfl_up((int)(unsigned)(incl >> 32), d, 64);
            if (lane >= d) incl += ((u64)hi << 32) | lo;
        }
        if (lane == 63) fsum[wave] = incl;
        __syncthreads();
        for (int v = 0; v < wave; ++v) incl += fsum[v];
        u64 below = incl - mine;
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            if (below < k && below + c[q] >= k) { chosen = (unsigned)(4 * t + q); k_next = k - below; }
            below += c[q];
        }
        __syncthreads();
        if (chosen == 0xFFFFFFFFu) {                 // the rank is always covered: never expected
            if (t == 0) S->g[0].gather_error = 1;
            return;
        }
        prefix = (prefix << w) | chosen;
        k = k_next;
        R = sh;
        __syncthreads();
    }
    if (t == 0) { sl.prefix = prefix; sl.k_rem = (i64)k; S->slot[0][s] = sl; }
}

// Workgroup = (column, quantile) slot: the slot's histogram from the row sums
// (thread = (bin, quarter of the rows)), the digit that holds the remaining
// rank, the extended prefix.
// After the first pass a slot's histogram is its own row: the workgroup adds up the slices itself.
__global__ __launch_bounds__(1024) void k_ttft_select(SelState* S, int pass, int P, int nq, const unsigned* __restrict__ rowsum,
                                                      const unsigned* __restrict__ slices, int nsl_pair, int nsl_cls)
{
    __shared__ u64 part[1024];
    __shared__ u64 wsum[4];
    const PassDigit dg = pass_digit(S->g[0], pass);
    if (dg.width <= 0) return;
    const int width = dg.width;
    const int s = blockIdx.x;
    SelSlot sl = S->slot[0][s];
    if (sl.done) return;
    const int col = s / nq;
    if (pass >= 1 && S->tb.on) {
        if (pass == 1) {
            const int b = S->tb.of_slot[s];
            const unsigned fill = S->tb.fill[b], cap = S->tb.cap[b];
            finish_from_list<true>(S, s, col, sl, slices + S->tb.base[b], fill < cap ? fill : cap, S->g[0].plan.shift[0]);
        }
        return;
    }
    if (pass >= 2 && gather_on(S->g[0])) {
        const unsigned nl = S->g[0].n_list;
        if (pass == 2) finish_from_list<false>(S, s, col, sl, slices, nl < TG_CAP ? nl : TG_CAP, S->g[0].plan.shift[1]);
        return;
    }
    const int nbins = 1 << width;                          // <= 256
    const int t = threadIdx.x & 255, q = threadIdx.x >> 8, lane = t & 63, wave = t >> 6;
    u64 mine = 0;
    if (t < nbins) {
        if (pass > 0) {
            const int nsl = S->tc.on ? nsl_cls : nsl_pair;
            const size_t step = (size_t)(P * nq) << width;
            const unsigned* src = slices + ((size_t)s << width) + t;
            unsigned a0 = 0, a1 = 0, a2 = 0, a3 = 0;
            int b = q;
            for (; b + 12 < nsl; b += 16) {
                a0 += src[(size_t)b * step]; a1 += src[(size_t)(b + 4) * step];
                a2 += src[(size_t)(b + 8) * step]; a3 += src[(size_t)(b + 12) * step];
            }
            for (; b < nsl; b += 4) a0 += src[(size_t)b * step];
            mine = (u64)a0 + a1 + a2 + a3;
        } else if (!S->tc.on) {
            if (q == 0) mine = rowsum[((size_t)col << width) + t];
        } else {                                           // device rows ub <= p, race rows ub > p
            const int p = S->tc.pos_of_col[col];
            for (int ub = q; ub <= P; ub += 4) mine += rowsum[((size_t)(ub <= p ? ub : P + 1 + ub) << width) + t];
        }
    }
    part[threadIdx.x] = mine;
    __syncthreads();
    mine = part[t] + part[256 + t] + part[512 + t] + part[768 + t];     // every quarter computes the same sums
    u64 incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        unsigned lo = (unsigned)__shfl_up((int)(unsigned)incl, d, 64);
        unsigned hi = (unsigned)__shfl_up((int)(unsigned)(incl >> 32), d, 64);
        if (lane >= d) incl += ((u64)hi << 32) | lo;
    }
    if (q == 0 && lane == 63) wsum[wave] = incl;
    __syncthreads();
    for (int w = 0; w < wave; ++w) incl += wsum[w];
    const u64 k = (u64)sl.k_rem;
    // the rank never exceeds the number of matching values: exactly one bin takes it
    if (q == 0 && t < nbins && incl >= k && incl - mine < k) {
        sl.k_rem = (i64)(k - (incl - mine));
        sl.prefix = (sl.prefix << width) | (unsigned)t;
        S->slot[0][s] = sl;
        // every value that still matches some slot after this pass is counted in that slot's bin
        if (pass == 1) atomicAdd((unsigned long long*)&S->g[0].gather_bound, (unsigned long long)mine);
    }
}

template <int G>
void launch_hist(const TraceView& v, const disco_policy* pol, int P, int nq, int pass, SelState* S, unsigned* slices,
                 unsigned bp, unsigned bc, unsigned char* ubytes, const unsigned* rowsum, hipStream_t stream)
{
    hipLaunchKernelGGL(k_ttft_hist<G>, dim3(bc + bp), dim3(DP_BLOCK), 0, stream, v, pol, P, nq, pass, S, slices, (int)bc,
                       ubytes, rowsum);
}

}  // namespace

void disco_launch_ttft_pass(const TraceView& v, const disco_policy* pol, int P, int nq, int pass, SelState* S,
                            unsigned* slices, unsigned* rowsum, unsigned char* ubytes, hipStream_t stream)
{
    i64 bp = ((v.n_req + 63) / 64 + DP_WAVES - 1) / DP_WAVES;
    if (bp < 1) bp = 1;
    if (bp > DP_MAX_BLOCKS) bp = DP_MAX_BLOCKS;
    i64 bc = (v.n_req + DP_BLOCK - 1) / DP_BLOCK;
    if (bc < 1) bc = 1;
    if (bc > TC_MAX_BLOCKS) bc = TC_MAX_BLOCKS;
    int g = 1;
    while (g < P) g <<= 1;
    switch (g) {
    case 1: launch_hist<1>(v, pol, P, nq, pass, S, slices, (unsigned)bp, (unsigned)bc, ubytes, rowsum, stream); break;
    case 2: launch_hist<2>(v, pol, P, nq, pass, S, slices, (unsigned)bp, (unsigned)bc, ubytes, rowsum, stream); break;
    case 4: launch_hist<4>(v, pol, P, nq, pass, S, slices, (unsigned)bp, (unsigned)bc, ubytes, rowsum, stream); break;
    case 8: launch_hist<8>(v, pol, P, nq, pass, S, slices, (unsigned)bp, (unsigned)bc, ubytes, rowsum, stream); break;
    case 16: launch_hist<16>(v, pol, P, nq, pass, S, slices, (unsigned)bp, (unsigned)bc, ubytes, rowsum, stream); break;
    case 32: launch_hist<32>(v, pol, P, nq, pass, S, slices, (unsigned)bp, (unsigned)bc, ubytes, rowsum, stream); break;
    default: launch_hist<64>(v, pol, P, nq, pass, S, slices, (unsigned)bp, (unsigned)bc, ubytes, rowsum, stream); break;
    }
    const int rows_pair = pass == 0 ? P : P * nq, rows_cls = pass == 0 ? 2 * (P + 1) : P * nq;
    const int rows_max = rows_pair > rows_cls ? rows_pair : rows_cls;
    if (pass == 0)          // the rows of the first pass are shared by many slots: summed once
        hipLaunchKernelGGL(k_ttft_reduce, dim3((unsigned)rows_max), dim3(1024), 0, stream, S, pass, rows_pair, rows_cls, (int)bp,
                           (int)bc, slices, rowsum);
    hipLaunchKernelGGL(k_ttft_select, dim3((unsigned)(P * nq)), dim3(1024), 0, stream, S, pass, P, nq, rowsum, slices, (int)bp,
                       (int)bc);
}
