// Closed-form policy solves of the dispatch controller on a resident trace
// (Sec. 4.2): Alg. 3 / Eq. 3 -- the length threshold that leaves the server
// the share b of the prompt tokens -- and Alg. 2 -- Phase 1: tail wait
// w_tail = F^-1(1 - min(alpha, b)); Phase 2: the remaining budget buys
// immediate device starts for the shortest prompts and one partial wait.
//
// The distributions are the trace's own: p(l) = requests per prompt length,
// F = empirical distribution of the server TTFT (nearest-rank inverse).  The
// sorted sweep over the length support of the paper becomes
//   1. the table of prompt-token mass by length and its suffix sums (the
//      kernels of the tabulated threshold search),
//   2. one thread per column that finds the last affordable length by binary
//      search in those sums -- all budget comparisons in exact 128-bit integer
//      arithmetic on the rational budget b and tail ratio alpha -- and the
//      ranks of the server TTFTs that become w_tail and the partial wait,
//   3. an exact multi-rank radix selection over the server TTFTs (four 8-bit
//      passes over the bit patterns; one LDS histogram row per distinct prefix
//      of the wanted ranks),
//   4. one thread per column writing the policy record.
#include <string.h>

#include "disco_launch.h"
#include "disco_state.h"
#include "disco_device.h"

namespace {

typedef unsigned __int128 u128;

constexpr int SQ_BLOCK = 1024;
constexpr int SQ_MAX_BLOCKS = 128;                 // slices of 128 rows x 256 bins x 4 B = 128 KB each
constexpr int SQ_STRIDE = 257;                     // skewed rows

struct SolveSlot { i64 k_rem; unsigned prefix; int live; };
struct SolveState {
    SolveSlot slot[2 * DISCO_MAX_COLS];            // slot 2c: tail wait of column c, 2c + 1: its partial wait
    disco_solve_out out[DISCO_MAX_COLS];
    disco_policy pol[DISCO_MAX_COLS];
};

struct SolveSpecs { disco_solve_spec s[DISCO_MAX_COLS]; };

// Mass of the prompts of length <= L (tokens): total - sum over lengths > L.
__device__ __forceinline__ u64 mass_upto(const u64* __restrict__ table, int nbins, int L)
{
    return L < 0 ? 0ull : table[0] - table[L + 1 < nbins ? L + 1 : nbins];
}

// Step 2 (thread = column).
__global__ void k_solve_plan(SolveSpecs specs, int n, i64 n_req, int nbins, const u64* __restrict__ table, SolveState* S)
{
    const int c = threadIdx.x;
    if (c >= n) return;
    const disco_solve_spec sp = specs.s[c];
    const u64 total = table[0];
    disco_policy p;
    memset(&p, 0, sizeof(p));
    p.mode = sp.mode; p.l_th = -1; p.l_mid = -1; p.w_mid = 0.0f; p.beta = INFINITY; p.w_tail = INFINITY;
    p.mig_mode = sp.mig_mode;
    disco_solve_out o;
    memset(&o, 0, sizeof(o));
    o.status = table[nbins] != 0ull ? 1 : 0;        // prompts longer than the table holds
    o.total_tokens = (i64)total;
    SolveSlot tail{0, 0u, 0}, mid{0, 0u, 0};
    const u64 bn = (u64)sp.b_num, bd = (u64)sp.b_den, an = (u64)sp.a_num, ad = (u64)sp.a_den;
    if (sp.mode == DISCO_MODE_SERVER_CONSTRAINED) {
        // Eq. 3, discrete: the smallest L with (tokens of the prompts of length >= L) <= b x (all tokens)
        const u128 budget = (u128)bn * (u128)total;
        int lo = 0, hi = nbins;                     // table[nbins] = lengths beyond the table
        while (lo < hi) {
            const int m = lo + (hi - lo) / 2;
            if ((u128)table[m] * (u128)bd <= budget) hi = m; else lo = m + 1;
        }
        p.l_th = lo;
        p.beta = INFINITY; p.w_tail = INFINITY;
        o.zero_wait_tokens = (i64)(total - table[lo]);      // tokens of the device-only prompts
    } else {
        // Phase 1: rank of w_tail = ceil((1 - min(alpha, b)) N)
        const bool b_le_a = bn * ad <= an * bd;
        const u64 mn = b_le_a ? bn : an, md = b_le_a ? bd : ad;
        i64 rank_tail = (i64)(((md - mn) * (u64)n_req + md - 1) / md);
        if (rank_tail > n_req) rank_tail = n_req;
        o.rank_tail = rank_tail;
        tail.k_rem = rank_tail; tail.live = rank_tail > 0;
        if (!b_le_a) {
            // Phase 2 in units of tokens / (a_den b_den): available = (b - alpha) total; a length costs (1 - alpha) mass
            const u128 avail = (u128)(bn * ad - an * bd) * (u128)total;
            const u64 K = (ad - an) * bd;
            int lo = -1, hi = nbins - 1;            // the largest L whose prefix of lengths is affordable
            while (lo < hi) {
                const int m = lo + (hi - lo + 1) / 2;
                if ((u128)K * (u128)mass_upto(table, nbins, m) <= avail) lo = m; else hi = m - 1;
            }
            const u64 zero_mass = mass_upto(table, nbins, lo);
            // snap to the last length that occurs: the smallest L with the same mass below it
            int a = -1, z = lo;
            while (a < z) {
                const int m = a + (z - a) / 2;
                if (mass_upto(table, nbins, m) == zero_mass) z = m; else a = m + 1;
            }
            p.l_th = zero_mass ? a : -1;
            o.zero_wait_tokens = (i64)zero_mass;
            // the next length that occurs gets the partial wait
            const u64 above = total - zero_mass;    // tokens of the longer prompts
            if (above > table[nbins]) {
                int x = lo + 1, y = nbins - 1;      // smallest L > lo with mass_upto(L) > zero_mass
                while (x < y) {
                    const int m = x + (y - x) / 2;
                    if (mass_upto(table, nbins, m) > zero_mass) y = m; else x = m + 1;
                }
                const u64 mass_mid = mass_upto(table, nbins, x) - zero_mass;
                p.l_mid = x;
                // (1 - alpha - F(w*)) mass = available left  <=>  F(w*) = (K mass - left) / (a_den b_den mass)
                const u128 left = avail - (u128)K * (u128)zero_mass;
                const u128 num = ((u128)K * (u128)mass_mid - left) * (u128)(u64)n_req;
                const u128 den = (u128)(ad * bd) * (u128)mass_mid;
                i64 k0 = 0, k1 = n_req;             // rank = ceil(F N): the smallest k with k den >= num
                while (k0 < k1) {
                    const i64 m = k0 + (k1 - k0) / 2;
                    if ((u128)(u64)m * den >= num) k1 = m; else k0 = m + 1;
                }
                o.rank_mid = k0;
                mid.k_rem = k0; mid.live = k0 > 0;
            }
        }
    }
    S->slot[2 * c] = tail;
    S->slot[2 * c + 1] = mid;
    S->out[c] = o;
    S->pol[c] = p;
}

// Step 3, histogram of one 8-bit digit.  Row r of the workgroup's LDS bins
// belongs to the r-th distinct prefix among the live slots; the slice written
// at the end has one row per slot (slots that share a prefix get copies).
__global__ __launch_bounds__(SQ_BLOCK) void k_sq_hist(const float* __restrict__ s, i64 n_req, int nslot, int pass,
                                                      const SolveState* S, unsigned* __restrict__ slices)
{
    __shared__ unsigned hist[2 * DISCO_MAX_COLS * SQ_STRIDE];
    __shared__ unsigned sprefix[2 * DISCO_MAX_COLS], dist[2 * DISCO_MAX_COLS];
    __shared__ int slive[2 * DISCO_MAX_COLS], first[2 * DISCO_MAX_COLS], rank[2 * DISCO_MAX_COLS], row_of[2 * DISCO_MAX_COLS];
    __shared__ int ndist;
    constexpr int NS = 2 * DISCO_MAX_COLS;
    const int t = threadIdx.x;
    const int shift = 24 - 8 * pass;
    if (t < NS) {
        const bool in = t < nslot;
        SolveSlot sl{0, 0u, 0};
        if (in) sl = S->slot[t];
        sprefix[t] = sl.prefix; slive[t] = in && sl.live; first[t] = in && sl.live; rank[t] = 0; row_of[t] = 0;
    }
    if (t == 0) ndist = 0;
    __syncthreads();
    for (int pr = t; pr < NS * NS; pr += SQ_BLOCK) {
        const int a = pr / NS, z = pr % NS;
        if (z < a && slive[z] && slive[a] && sprefix[z] == sprefix[a]) first[a] = 0;
    }
    __syncthreads();
    for (int pr = t; pr < NS * NS; pr += SQ_BLOCK) {
        const int a = pr / NS, o = pr % NS;
        if (first[a] && first[o] && sprefix[o] < sprefix[a]) atomicAdd(&rank[a], 1);
    }
    __syncthreads();
    if (t < NS && first[t]) { dist[rank[t]] = sprefix[t]; atomicAdd(&ndist, 1); }
    for (int pr = t; pr < NS * NS; pr += SQ_BLOCK) {
        const int a = pr / NS, o = pr % NS;
        if (first[a] && slive[o] && sprefix[o] == sprefix[a]) row_of[o] = rank[a];
    }
    __syncthreads();
    const int nd = ndist;
    if (nd == 0) return;                            // nothing left to select (uniform)
    for (int i = t; i < nd * SQ_STRIDE; i += SQ_BLOCK) hist[i] = 0u;
    __syncthreads();
    for (i64 i = (i64)blockIdx.x * SQ_BLOCK + t; i < n_req; i += (i64)gridDim.x * SQ_BLOCK) {
        const unsigned key = f2u(s[i]);
        const unsigned hi = pass == 0 ? 0u : key >> (shift + 8);
        int lo_i = 0, hi_i = nd;                    // first distinct prefix >= hi
        while (lo_i < hi_i) {
            const int m = (lo_i + hi_i) >> 1;
            if (dist[m] < hi) lo_i = m + 1; else hi_i = m;
        }
        if (lo_i < nd && dist[lo_i] == hi) atomicAdd(&hist[lo_i * SQ_STRIDE + ((key >> shift) & 255u)], 1u);
    }
    __syncthreads();
    unsigned* mine = slices + (size_t)blockIdx.x * ((size_t)nslot << 8);
    for (int i = t; i < nslot << 8; i += SQ_BLOCK) {
        const int sl = i >> 8;
        mine[i] = slive[sl] ? hist[row_of[sl] * SQ_STRIDE + (i & 255)] : 0u;
    }
}

// Step 3, digit choice: workgroup = slot, thread = (bin, quarter of the slices).
__global__ __launch_bounds__(1024) void k_sq_select(int nslot, int nslices, const unsigned* __restrict__ slices, SolveState* S)
{
    __shared__ u64 part[1024];
    __shared__ u64 wsum[4];
    const int sidx = blockIdx.x, t = threadIdx.x & 255, q = threadIdx.x >> 8, lane = t & 63, wave = t >> 6;
    SolveSlot sl = S->slot[sidx];
    if (!sl.live) return;
    const size_t step = (size_t)nslot << 8;
    const unsigned* src = slices + ((size_t)sidx << 8) + t;
    unsigned a0 = 0, a1 = 0, a2 = 0, a3 = 0;
    int b = q;
    for (; b + 12 < nslices; b += 16) {
        a0 += src[(size_t)b * step]; a1 += src[(size_t)(b + 4) * step];
        a2 += src[(size_t)(b + 8) * step]; a3 += src[(size_t)(b + 12) * step];
    }
    for (; b < nslices; b += 4) a0 += src[(size_t)b * step];
    part[threadIdx.x] = (u64)a0 + a1 + a2 + a3;
    __syncthreads();
    const u64 mine = part[t] + part[256 + t] + part[512 + t] + part[768 + t];     // every quarter computes the same sums
    u64 incl = mine;
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        const unsigned lo = (unsigned)__shfl_up((int)(unsigned)incl, d, 64);
        const unsigned hi = (unsigned)__shfl_up((int)(unsigned)(incl >> 32), d, 64);
        if (lane >= d) incl += ((u64)hi << 32) | lo;
    }
    if (q == 0 && lane == 63) wsum[wave] = incl;
    __syncthreads();
    for (int w = 0; w < wave; ++w) incl += wsum[w];
    const u64 k = (u64)sl.k_rem;
    if (q == 0 && incl >= k && incl - mine < k) {   // exactly one bin holds the remaining rank
        sl.k_rem = (i64)(k - (incl - mine));
        sl.prefix = (sl.prefix << 8) | (unsigned)t;
        S->slot[sidx] = sl;
    }
}

// Step 4 (thread = column).
__global__ void k_solve_final(int n, const SolveState* S, disco_policy* pol_out, disco_solve_out* out)
{
    const int c = threadIdx.x;
    if (c >= n) return;
    disco_policy p = S->pol[c];
    if (p.mode == DISCO_MODE_DEVICE_CONSTRAINED) {
        const SolveSlot tail = S->slot[2 * c], mid = S->slot[2 * c + 1];
        p.w_tail = tail.live ? u2f(tail.prefix) : 0.0f;      // rank 0: F^-1(0) = 0
        p.w_mid = mid.live ? u2f(mid.prefix) : 0.0f;
    }
    pol_out[c] = p;
    if (out) out[c] = S->out[c];
}

__global__ void k_solve_init(u64* other) { if (threadIdx.x == 0) *other = 0ull; }

}  // namespace

size_t disco_solve_state_bytes(void) { return sizeof(SolveState); }

void disco_launch_solve(const TraceView& v, const disco_solve_spec* spec, int n, void* state, u64* table, u64* other,
                        unsigned* scratch, size_t scratch_bytes, disco_policy* pol_out, disco_solve_out* out,
                        hipStream_t stream)
{
    SolveState* S = (SolveState*)state;
    const int nbins = disco_search_table_max_bins();
    hipLaunchKernelGGL(k_solve_init, dim3(1), dim3(64), 0, stream, other);
    disco_launch_len_table(v, nbins, scratch, scratch_bytes, table, other, stream);
    SolveSpecs t;
    memset(&t, 0, sizeof(t));
    memcpy(t.s, spec, sizeof(disco_solve_spec) * (size_t)n);
    hipLaunchKernelGGL(k_solve_plan, dim3(1), dim3(64), 0, stream, t, n, v.n_req, nbins, table, S);
    const int nslot = 2 * n;
    i64 blocks = (v.n_req + SQ_BLOCK - 1) / SQ_BLOCK;
    const i64 fit = (i64)(scratch_bytes / (((size_t)nslot << 8) * sizeof(unsigned)));
    if (blocks > fit) blocks = fit;
    if (blocks > SQ_MAX_BLOCKS) blocks = SQ_MAX_BLOCKS;
    if (blocks < 1) blocks = 1;
    for (int pass = 0; pass < 4; ++pass) {
        hipLaunchKernelGGL(k_sq_hist, dim3((unsigned)blocks), dim3(SQ_BLOCK), 0, stream, v.s, v.n_req, nslot, pass, S, scratch);
        hipLaunchKernelGGL(k_sq_select, dim3((unsigned)nslot), dim3(1024), 0, stream, nslot, (int)blocks, scratch, S);
    }
    hipLaunchKernelGGL(k_solve_final, dim3(1), dim3(64), 0, stream, n, S, pol_out, out);
}
