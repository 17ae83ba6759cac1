// Device-resident state shared by the passes of libdisco and the helpers that
// advance it at the end of a pass (last-ticket workgroup).
#pragma once
#include "disco_common.h"
#include "disco_device.h"

struct PolTable { disco_policy p[DISCO_MAX_COLS]; };

struct SearchState {
    double lo, hi, target;
    int32_t which_param, which_acc, step, n_steps;
};
struct SpecTable { SearchState s[DISCO_MAX_COLS]; };

// Bisection of a budget search (Sec. 4.2: the threshold, wait or ramp slope that meets the constrained
// endpoint's budget) on the bracket [lo, hi] of its state: the parameter evaluated for a bracket is its midpoint,
// the answer once the steps are used up its feasible end hi.  prm = DISCO_PARAM_*: l_th is bisected in integers,
// w_tail and beta (Eq. 1's ramp slope, the unknown of Eq. 2) in fp32.
__device__ __forceinline__ void search_set_value(int prm, float x, disco_policy& p)
{
    if (prm == DISCO_PARAM_W_TAIL) p.w_tail = x; else p.beta = x;
}
__device__ __forceinline__ void search_set_mid(int prm, double lo, double hi, disco_policy& p)
{
    if (prm == DISCO_PARAM_L_TH) { const int l = (int)lo, h = (int)hi; p.l_th = l + (h - l) / 2; }
    else search_set_value(prm, 0.5f * ((float)lo + (float)hi), p);
}
__device__ __forceinline__ void search_set_answer(int prm, double hi, disco_policy& p)
{
    if (prm == DISCO_PARAM_L_TH) p.l_th = (int)hi; else search_set_value(prm, (float)hi, p);
}
__device__ __forceinline__ double search_param(int prm, const disco_policy& p)
{
    return prm == DISCO_PARAM_L_TH ? (double)p.l_th : (prm == DISCO_PARAM_W_TAIL ? (double)p.w_tail : (double)p.beta);
}
// above: the accumulator at `mid` exceeds the target
__device__ __forceinline__ void search_halve(int prm, double& lo, double& hi, double mid, bool above)
{
    if (prm != DISCO_PARAM_L_TH) { if (above) lo = mid; else hi = mid; }
    else if (lo < hi) { if (above) lo = mid + 1.0; else hi = mid; }
}
// The parameters of the next `depth` (<= 3) levels of the bisection below the bracket of `st`, as policy records
// in heap order (node 1 = the midpoint of the bracket, node 2n = after "not above" at node n, 2n + 1 = after
// "above"): dst[0 .. 2^depth - 1).  A search whose steps are used up gets copies of its answer.
__device__ inline void search_write_candidates(const SearchState& st, const disco_policy& templ, disco_policy* dst, int depth)
{
    const int prm = st.which_param;
    const int M = (1 << depth) - 1;
    double lo[8], hi[8];
    lo[1] = st.lo; hi[1] = st.hi;
    for (int node = 1; node <= M; ++node) {
        disco_policy p = templ;
        if (st.step >= st.n_steps) search_set_answer(prm, st.hi, p);
        else search_set_mid(prm, lo[node], hi[node], p);
        dst[node - 1] = p;
        if (2 * node + 1 <= M) {
            const double mid = search_param(prm, p);
            lo[2 * node] = lo[node]; hi[2 * node] = hi[node];
            search_halve(prm, lo[2 * node], hi[2 * node], mid, false);
            lo[2 * node + 1] = lo[node]; hi[2 * node + 1] = hi[node];
            search_halve(prm, lo[2 * node + 1], hi[2 * node + 1], mid, true);
        }
    }
}

// Order-statistic selection: most-significant-digit-first radix histograms
// over key = bits(value) - minb (non-negative floats order like their bit
// patterns).  Pass p looks at `width[p]` bits at `shift[p]`.
enum { DISCO_MAX_PASS = 6 };
struct SelPlan { int npass; int shift[DISCO_MAX_PASS]; int width[DISCO_MAX_PASS]; int pad; };
// gather_bound: after the second pass, an upper bound of the values that still match some slot's prefix; when it
// is small they are collected in a list (n_list entries) and the remaining digits are decided from the list.
struct SelGlobal { unsigned minb, maxb; SelPlan plan; u64 gather_bound; unsigned n_list; int gather_error; };
struct SelSlot { unsigned prefix; int done; i64 k_rem; i64 rank; i64 M; };
// TBT selection: a timeline is histogrammed once per *class* = set of policy
// columns that use it (for threshold- or wait-ordered tables the sets are
// nested, so there are at most P + 1 of them), not once per column.  Keys are
// the raw 31-bit patterns of the gaps.  The digit of each pass is sized on the
// device from the number of classes and of distinct prefixes still alive.
enum { DISCO_MAX_CLS = 64, DISCO_CLS_SLOTS = 256, DISCO_MAX_GRP = 4, DISCO_TBT_MAX_PASS = 6,
       DISCO_TBT_REGULAR_PASS = 2,    // passes that normally decide every slot (the later ones are spare)
       DISCO_TL_HIST_WORDS = 16384,   // LDS bins of a timeline workgroup (64 KB: two workgroups per CU)
       DISCO_GHIST_WORDS = 262144,    // device-wide bins (1 MB)
       DISCO_PP_NMAX = 4096,          // pure-pacing timelines up to this length are histogrammed analytically
       DISCO_DELAY_BINS = 8192 };     // counts of delayed tokens per migrated request, per column (last bin: that or more)
struct TlSel {
    u64 cls_mask[DISCO_MAX_CLS];   // column set of each class, 0 = free
    u64 walk_mask;                 // classes with a timeline whose tokens have to be walked
    int ncls, nwalk;
    int fallback;                  // 1: one histogram per (column, quantile) slot instead of per class
    int error;                     // a column set could not be placed (never expected)
    int left;                      // undecided key bits
    int shift, width;              // digit of the pass about to run (width 0: finished)
    int G;                         // distinct prefixes among the live slots
    unsigned grp_prefix[DISCO_MAX_GRP];
    int slot_grp[DISCO_MAX_SLOTS]; // prefix group of each live slot, -1 otherwise
    // Window mode: keys are offsets from key_lo, clamped to 2^window ("outside", never counted).  Gaps sit just
    // above the pacing interval, so a 21-bit window above it holds the usual order statistics and two passes
    // decide them; a rank that falls outside (or into the clamped bottom bin) restarts the selection on raw keys.
    unsigned key_lo;
    int window;                    // key bits of the window, 0 = raw 31-bit keys
    int restart;
    unsigned nlist;                // requests with a timeline whose tokens are walked: entries at the front of the walk list
    unsigned nlist_back;           // ... and entries at its back (the short requests, see walk_list_entry)
    unsigned pad2;
    // device-wide hash table of the column sets (classification): every workgroup enters its distinct sets, the last
    // one numbers them; zeroed when a selection starts
    u64 gslot[DISCO_CLS_SLOTS];
    unsigned gwalk[DISCO_CLS_SLOTS];
    int goverflow;
    int pad3;
    signed char cls_slot[DISCO_MAX_CLS];     // row of a walked class in the workgroups' LDS histogram, -1 otherwise
    unsigned char slot_cls[DISCO_MAX_CLS];   // class of an LDS row
};
// TTFT selection by classes: set when every column is a length-threshold column (Alg. 3).
struct TtftCls {
    int on;
    int sorted_lth[DISCO_MAX_COLS];              // thresholds in ascending order
    unsigned char pos_of_col[DISCO_MAX_COLS];    // position of a column in that order
    unsigned char col_of_pos[DISCO_MAX_COLS];
    int pad[3];
};
// TTFT selection by classes, after the first pass: when all values that carry the first digit of some live slot
// fit the candidate list, the second pass sorts them into buckets (one per distinct digit, named by the smallest
// slot that has it) and every slot finishes its remaining digits from its bucket.  The workgroups of the second
// pass all derive the same plan from the row sums; the first one stores it here for the select kernel.
struct TtftBuckets {
    int on;
    int pad;
    unsigned base[DISCO_MAX_SLOTS];          // first entry of the bucket in the list (multiple of 4)
    unsigned cap[DISCO_MAX_SLOTS];           // entries it can take: the values of the first pass with that digit
    unsigned fill[DISCO_MAX_SLOTS];          // entries written
    int of_slot[DISCO_MAX_SLOTS];            // bucket of a slot, -1: none
};
struct SelState { SelGlobal g[2]; SelSlot slot[2][DISCO_MAX_SLOTS]; TlSel tl; TtftCls tc; TtftBuckets tb; };   // [0] TTFT, [1] TBT

// Device-wide totals are kept in DISCO_NCOPY copies (workgroup b adds into copy b % DISCO_NCOPY) so that
// the atomics of different workgroups do not all queue up on one cache line.
enum { DISCO_NCOPY = 16 };
struct DispPartial { u64 s_pre, d_pre, d_dec, n_tot, started, won; double ttft_sum; unsigned minb, maxb; };
struct MigPartial { u64 s_dec, d_dec, d_repre, migrated, tbt_count; double tlast_sum; u64 pad[2]; };
static_assert(sizeof(DispPartial) == 64 && sizeof(MigPartial) == 64, "partials are 64 bytes");
static_assert(sizeof(disco_accum) == 128 && sizeof(disco_stats) == 256 && sizeof(disco_policy) == 32, "ABI sizes");

// 64-byte partials are parked in LDS field by field (structure of arrays):
// consecutive threads then touch consecutive 8-byte words and the accesses
// are free of bank conflicts, which a 64-byte stride would serialise 32-fold.
template <class T>
__device__ __forceinline__ void lds_put(u64* sh, int cap, int idx, const T& v)
{
    static_assert(sizeof(T) == 64, "partials are 64 bytes");
    const u64* w = reinterpret_cast<const u64*>(&v);
#pragma unroll
    for (int f = 0; f < 8; ++f) sh[f * cap + idx] = w[f];
}
template <class T>
__device__ __forceinline__ T lds_get(const u64* sh, int cap, int idx)
{
    T v;
    u64* w = reinterpret_cast<u64*>(&v);
#pragma unroll
    for (int f = 0; f < 8; ++f) w[f] = sh[f * cap + idx];
    return v;
}

// Last-ticket test: true in every thread of the workgroup that finishes last.
__device__ __forceinline__ bool take_last_ticket(unsigned* ticket)
{
    __shared__ int is_last;
    __syncthreads();                       // the workgroup's writes are ordered before thread 0 ...
    if (threadIdx.x == 0) {
        __threadfence();                   // ... which releases them at device scope (one fence per workgroup)
        unsigned t = atomicAdd(ticket, 1u);
        is_last = (t == gridDim.x - 1);
    }
    __syncthreads();
    bool last = is_last != 0;
    if (last) __threadfence();
    return last;
}
