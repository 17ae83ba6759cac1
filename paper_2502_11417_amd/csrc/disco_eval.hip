// Evaluation kernels and entry points of libdisco: dispatch, token timelines
// with lag-triggered migration, order-statistic selection, budget search.
//
// Work decomposition
//   dispatch-type passes: a wave holds up to 64 policy columns in its lanes
//     and walks the requests in batches; per-column totals stay in registers
//     until the end of the kernel and are then added into device-wide totals.
//   timeline passes: one wave per request, four tokens per lane, 256-token
//     chunks with a carried running maximum.
//   a sequence of passes (budget search, radix selection) advances its state
//     on the device, so it needs no host round trip.
#include <math.h>
#include <stdio.h>
#include <string.h>

#include <mutex>

#include "disco_launch.h"
#include "disco_state.h"

namespace {

// The timeline totals follow the dispatch totals in the same workspace region.
__host__ __device__ inline MigPartial* tl_totals(u64* totals)
{
    return reinterpret_cast<MigPartial*>(totals + DISCO_NCOPY * 64 * 8);
}

// Start of a selection (all threads of one workgroup): one thread per slot: rank from (num, den, M), empty
// prefix; plan of the passes.
struct SelInit { SelState* S; int nq; disco_quantile q[4]; const disco_accum* acc; i64 n_req; int with_tbt; };

__device__ void select_init(const SelInit& si, int which, int P, const disco_policy* pol)
{
    SelState* S = si.S;
    const int nq = si.nq;
    const disco_accum* acc = si.acc;
    const i64 n_req = si.n_req;
    const disco_quantile qs[4] = {si.q[0], si.q[1], si.q[2], si.q[3]};
    __shared__ unsigned smin, smax;
    __shared__ int all_thresholds;
    if (threadIdx.x == 0) { smin = 0xFFFFFFFFu; smax = 0u; all_thresholds = 1; }
    __syncthreads();
    if (which == 0) {
        // a table of length-threshold columns (Alg. 3) is selected by classes: thresholds in ascending order
        const int t = threadIdx.x;
        __shared__ int lth_s[DISCO_MAX_COLS];
        if (t < P) {
            if (pol[t].mode != DISCO_MODE_SERVER_CONSTRAINED) all_thresholds = 0;
            lth_s[t] = pol[t].l_th;
        }
        __syncthreads();
        if (t < P) {
            const int lth = lth_s[t];
            int rank = 0;
            for (int k = 0; k < P; ++k) rank += (lth_s[k] < lth || (lth_s[k] == lth && k < t)) ? 1 : 0;
            S->tc.sorted_lth[rank] = lth;
            S->tc.col_of_pos[rank] = (unsigned char)t;
            S->tc.pos_of_col[t] = (unsigned char)rank;
        }
        __syncthreads();
        if (t == 0) { S->tc.on = all_thresholds; S->tb.on = 0; S->tb.pad = 0; }
        if (t < DISCO_MAX_SLOTS) { S->tb.fill[t] = 0u; S->tb.of_slot[t] = -1; }
    }
    if (which == 0 && (int)threadIdx.x < P) {
        atomicMin(&smin, acc[threadIdx.x].ttft_min_bits);
        atomicMax(&smax, acc[threadIdx.x].ttft_max_bits);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        SelGlobal g;
        if (which == 0) {
            g.minb = smin <= smax ? smin : 0u;
            g.maxb = smin <= smax ? smax : 0u;
            unsigned range = g.maxb - g.minb;
            int left = range ? 32 - __clz(range) : 0;
            SelPlan pl;
            pl.npass = 0; pl.pad = 0;
            for (int i = 0; i < DISCO_MAX_PASS; ++i) { pl.shift[i] = 0; pl.width[i] = 0; }
            while (left > 0) {
                int wd = left < 8 ? left : 8;
                pl.width[pl.npass] = wd; pl.shift[pl.npass] = left - wd;
                left -= wd; pl.npass += 1;
            }
            g.plan = pl;
            g.gather_bound = 0ull; g.n_list = 0u; g.gather_error = 0;
        } else {                      // TBT: raw keys; the passes are planned on the device (TlSel)
            g.minb = 0u; g.maxb = 0x7FFFFFFFu;
            g.gather_bound = 0ull; g.n_list = 0u; g.gather_error = 0;
            g.plan.npass = 0; g.plan.pad = 0;
            for (int i = 0; i < DISCO_MAX_PASS; ++i) { g.plan.shift[i] = 0; g.plan.width[i] = 0; }
            TlSel& tl = S->tl;
            tl.ncls = 0; tl.nwalk = 0; tl.walk_mask = 0ull; tl.fallback = 0; tl.error = 0; tl.left = 31; tl.shift = 0; tl.width = 0; tl.G = 0;
            tl.key_lo = 0u; tl.window = 0; tl.restart = 0;
            for (int i = 0; i < DISCO_MAX_GRP; ++i) tl.grp_prefix[i] = 0u;
        }
        S->g[which] = g;
    }
    if (which == 1) {
        for (int i = threadIdx.x; i < DISCO_MAX_CLS; i += blockDim.x) S->tl.cls_mask[i] = 0ull;
        for (int i = threadIdx.x; i < DISCO_CLS_SLOTS; i += blockDim.x) { S->tl.gslot[i] = 0ull; S->tl.gwalk[i] = 0u; }
        if (threadIdx.x == 0) S->tl.goverflow = 0;
        for (int i = threadIdx.x; i < DISCO_MAX_SLOTS; i += blockDim.x) S->tl.slot_grp[i] = -1;
    }
    for (int s = threadIdx.x; s < P * nq; s += blockDim.x) {
        int c = s / nq, qi = s % nq;
        i64 M = which ? acc[c].tbt_count : n_req;
        SelSlot sl;
        sl.M = M;
        i64 k = M > 0 ? ((i64)qs[qi].num * M + qs[qi].den - 1) / qs[qi].den : 0;
        if (M > 0 && k < 1) k = 1;
        if (k > M) k = M;
        sl.rank = k; sl.k_rem = k; sl.prefix = 0u; sl.done = (M <= 0);
        S->slot[which][s] = sl;
    }
}


// Staging of the policy table (wave 0); all 1024 threads also put the tickets and the per-column totals that
// the workgroups of a pass add into at their identity: the dispatch totals (8 words per column and copy,
// word-major; word 7 = {min bits, max bits}) and, behind them, the timeline totals (all zero).
constexpr int STAGE_THREADS = 1024;
__device__ inline void reset_totals(u64* totals)
{
    constexpr int DISP_WORDS = 8 * DISCO_NCOPY * 64, TL_WORDS = DISCO_NCOPY * 64 * (int)(sizeof(MigPartial) / 8);
    for (int w = threadIdx.x; w < DISP_WORDS + TL_WORDS; w += STAGE_THREADS)
        totals[w] = (w >= 7 * DISCO_NCOPY * 64 && w < DISP_WORDS) ? 0x00000000FFFFFFFFull : 0ull;
}

// With a selection state (si.S), the TTFT selection of the statistics (and, if asked, the TBT selection) is started
// in the same launch.
__global__ __launch_bounds__(STAGE_THREADS) void k_store_policies(PolTable t, int P, disco_policy* dst, unsigned* tickets, u64* totals,
                                                                  SelInit si)
{
    const int i = threadIdx.x;
    if (i < 64) {
        if (i < P) dst[i] = t.p[i];
        const bool any_buffer = __ballot(i < P && t.p[i < P ? i : 0].mig_mode == DISCO_MIG_BUFFER) != 0ull;
        tickets[i] = (i == DISCO_FLAG_BUFFER && any_buffer) ? 1u : 0u;
    }
    reset_totals(totals);
    if (si.S) {
        __syncthreads();                       // the staged table is read back by this workgroup
        select_init(si, 0, P, dst);
        if (si.with_tbt) {
            __syncthreads();
            select_init(si, 1, P, dst);
        }
    }
}

__global__ __launch_bounds__(STAGE_THREADS) void k_copy_policies(const disco_policy* src, int P, disco_policy* dst, unsigned* tickets, u64* totals,
                                                                 SelInit si)
{
    const int i = threadIdx.x;
    if (i < 64) {
        if (i < P) dst[i] = src[i];
        const bool any_buffer = __ballot(i < P && src[i < P ? i : 0].mig_mode == DISCO_MIG_BUFFER) != 0ull;
        tickets[i] = (i == DISCO_FLAG_BUFFER && any_buffer) ? 1u : 0u;
    }
    reset_totals(totals);
    if (si.S) {
        __syncthreads();                       // the staged table is read back by this workgroup
        select_init(si, 0, P, dst);
        if (si.with_tbt) {
            __syncthreads();
            select_init(si, 1, P, dst);
        }
    }
}

// ----------------------------------------------------------------- select --
// TTFT: key = bits - min_bits over nb = bit length of (max_bits - min_bits)
// bits, 8 bits per pass (up to 128 (column, quantile) slots of 256 bins in
// LDS).  TBT: the plan comes from the host (raw 31-bit keys).


// ------------------------------------------------------------ final stats --

// Order statistics of the delayed tokens per migrated request (all threads of a workgroup, column c): the counts
// by number of delayed tokens come from the first histogram pass of the timelines with a buffer hand-off;
// migrations of the lag trigger have none and count as zeros.  Nearest rank, like the other order statistics.
// dq[qi] keeps its value for a column without migrations.
__device__ void delay_quantiles(int c, int nq, const disco_quantile* qs, const disco_accum* acc, const unsigned* __restrict__ dhist,
                                u64* part /* LDS, 256 */, float* dq /* LDS */)
{
    constexpr int PER = DISCO_DELAY_BINS / 256;
    const int t = threadIdx.x;
    const i64 M = acc[c].n_migrated;
    if (M <= 0) return;                                  // (the same answer in every thread)
    const unsigned* row = dhist + (size_t)c * DISCO_DELAY_BINS;
    unsigned v[PER];
    u64 mine = 0;
#pragma unroll
    for (int k = 0; k < PER; ++k) { v[k] = row[t * PER + k]; mine += v[k]; }
    part[t] = mine;
    __syncthreads();
    for (int d = 1; d < 256; d <<= 1) {                  // inclusive prefix sums of the per-thread totals
        const u64 o = t >= d ? part[t - d] : 0;
        __syncthreads();
        part[t] += o;
        __syncthreads();
    }
    const u64 counted = part[255];
    const u64 zeros = (u64)M > counted ? (u64)M - counted : 0;      // hand-offs without a count: no delayed token
    if (t == 0) v[0] += (unsigned)zeros;
    const u64 below = t > 0 ? part[t - 1] + zeros : 0;               // migrated requests with fewer delayed tokens than t * PER
    for (int qi = 0; qi < nq; ++qi) {
        i64 k = ((i64)qs[qi].num * M + qs[qi].den - 1) / qs[qi].den;
        if (k < 1) k = 1;
        if (k > M) k = M;
        u64 cum = below;
#pragma unroll
        for (int b = 0; b < PER; ++b) {
            if (cum < (u64)k && cum + v[b] >= (u64)k) dq[qi] = (float)(t * PER + b);
            cum += v[b];
        }
    }
}

// The record of a column from its accumulators and the selections' results.  With delayed-token order statistics
// to work out (timelines and quantiles asked for): workgroup = column, 256 threads; otherwise one workgroup,
// thread = column.
__global__ __launch_bounds__(256) void k_stats_final(int P, int nq, i64 n_req, disco_cost_params cost, int with_tl,
                                                     const disco_accum* acc, const SelState* S, disco_quantile q0,
                                                     disco_quantile q1, disco_quantile q2, disco_quantile q3,
                                                     const unsigned* __restrict__ dhist, disco_stats* out)
{
    __shared__ u64 part[256];
    __shared__ float dq[DISCO_MAX_Q];
    const bool per_column = with_tl && nq > 0;
    const int c = per_column ? blockIdx.x : threadIdx.x;
    if (threadIdx.x < DISCO_MAX_Q) dq[threadIdx.x] = NAN;
    __syncthreads();
    if (per_column) {
        const disco_quantile qs[4] = {q0, q1, q2, q3};
        delay_quantiles(c, nq, qs, acc, dhist, part, dq);
        __syncthreads();
        if (threadIdx.x != 0) return;
    } else if (c >= P) {
        return;
    }
    const disco_accum a = acc[c];
    disco_stats st;
    memset(&st, 0, sizeof(st));
    st.n_req = n_req;
    st.s_pre = a.s_pre + (with_tl ? a.m_s_repre : 0);
    st.d_pre = a.d_pre + (with_tl ? a.m_d_repre : 0);
    st.s_dec = with_tl ? a.m_s_dec : a.s_dec;
    st.d_dec = with_tl ? a.m_d_dec : a.d_dec;
    st.n_dev_started = a.n_dev_started;
    st.n_dev_win = a.n_dev_win;
    st.n_migrated = with_tl ? a.n_migrated : 0;
    st.tbt_count = with_tl ? a.tbt_count : 0;
    st.mean_ttft = a.ttft_sum / (double)n_req;                       // 0/0 = NaN for an empty batch
    st.mean_tbt = with_tl ? a.tlast_sum / (double)a.tbt_count : NAN;  // telescoped sum of gaps
    st.mean_delay_num = (with_tl && a.n_migrated > 0) ? (double)a.delay_sum / (double)a.n_migrated : NAN;
    st.server_cost = server_cost_of(cost, st.s_pre, st.s_dec);
    st.device_energy = device_energy_of(cost, st.d_pre, st.d_dec);
    st.device_cost = cost.lambda * st.device_energy;
    st.total_cost = st.server_cost + st.device_cost;
    for (int qi = 0; qi < DISCO_MAX_Q; ++qi) {
        st.ttft_q[qi] = NAN; st.tbt_q[qi] = NAN; st.delay_q[qi] = dq[qi];
        if (qi < nq) {
            const SelSlot s0 = S->slot[0][c * nq + qi];
            st.ttft_rank[qi] = s0.rank;
            if (s0.M > 0 && !S->g[0].gather_error) st.ttft_q[qi] = u2f(S->g[0].minb + s0.prefix);
            if (with_tl) {
                const SelSlot s1 = S->slot[1][c * nq + qi];
                st.tbt_rank[qi] = s1.rank;
                if (s1.M > 0 && !S->tl.error && S->tl.left == 0) st.tbt_q[qi] = u2f(s1.prefix + S->tl.key_lo);
            }
        }
    }
    out[c] = st;
}

// Mean over the runs of a group of columns: floating-point fields in fp64, summed in run order; integer
// totals summed; ranks taken from the first run.
__global__ void k_average_runs(const disco_stats* __restrict__ in, int groups, int runs, disco_stats* __restrict__ out)
{
    const int g = blockIdx.x * blockDim.x + threadIdx.x;
    if (g >= groups) return;
    const disco_stats* r = in + (size_t)g * runs;
    disco_stats o;
    memset(&o, 0, sizeof(o));
    double d[7] = {0, 0, 0, 0, 0, 0, 0}, q[2 * DISCO_MAX_Q];
    for (int k = 0; k < 2 * DISCO_MAX_Q; ++k) q[k] = 0.0;
    for (int k = 0; k < DISCO_MAX_Q; ++k) { o.ttft_rank[k] = r[0].ttft_rank[k]; o.tbt_rank[k] = r[0].tbt_rank[k]; }
    for (int j = 0; j < runs; ++j) {
        const disco_stats s = r[j];
        d[0] += s.mean_ttft; d[1] += s.mean_tbt; d[2] += s.server_cost; d[3] += s.device_energy;
        d[4] += s.device_cost; d[5] += s.total_cost; d[6] += s.mean_delay_num;
        o.s_pre += s.s_pre; o.s_dec += s.s_dec; o.d_pre += s.d_pre; o.d_dec += s.d_dec;
        o.n_req += s.n_req; o.tbt_count += s.tbt_count; o.n_migrated += s.n_migrated;
        o.n_dev_started += s.n_dev_started; o.n_dev_win += s.n_dev_win;
        for (int k = 0; k < DISCO_MAX_Q; ++k) { q[k] += (double)s.ttft_q[k]; q[DISCO_MAX_Q + k] += (double)s.tbt_q[k]; }
    }
    const double n = (double)runs;
    o.mean_ttft = d[0] / n; o.mean_tbt = d[1] / n; o.server_cost = d[2] / n; o.device_energy = d[3] / n;
    o.device_cost = d[4] / n; o.total_cost = d[5] / n; o.mean_delay_num = d[6] / n;
    for (int k = 0; k < DISCO_MAX_Q; ++k) { o.ttft_q[k] = (float)(q[k] / n); o.tbt_q[k] = (float)(q[DISCO_MAX_Q + k] / n); }
    out[g] = o;
}

// ----------------------------------------------------------- search setup --

// Brackets of the searches; `pol` holds their templates on entry.  depth > 0: the templates move to `templ`
// and `pol` gets the candidate columns of the first bisection pass (2^depth - 1 per search); depth 0 (tabulated
// threshold search): `pol` keeps one record per search with the first midpoint.
__global__ void k_search_init(SpecTable t, int n, SearchState* st, disco_policy* pol, disco_policy* templ, int depth)
{
    const int c = threadIdx.x;
    SearchState s;
    disco_policy p;
    if (c < n) {
        s = t.s[c];
        p = pol[c];
        if (s.which_param == DISCO_PARAM_L_TH) { s.lo = (int)s.lo; s.hi = (int)s.hi; }
        else { s.lo = (double)(float)s.lo; s.hi = (double)(float)s.hi; }
        s.step = 0;
        st[c] = s;
    }
    __syncthreads();                        // all templates have been read
    if (c >= n) return;
    if (depth > 0) {
        templ[c] = p;
        search_write_candidates(s, p, &pol[c * ((1 << depth) - 1)], depth);
    } else {
        search_set_mid(s.which_param, s.lo, s.hi, p);
        pol[c] = p;
    }
}

// ------------------------------------------------------------- host side --

thread_local char g_hip_error[256] = "";

TraceView view_of(const disco_trace* t)
{
    TraceView v;
    v.n_req = t->n_req;
    v.l = t->prompt_len; v.n = t->output_len; v.s = t->srv_ttft; v.tbt = t->srv_tbt;
    v.k = t->dev_pre_spt; v.g = t->dev_dec_spt;
    v.off = t->tok_arr ? t->tok_off : nullptr;
    v.arr = t->tok_arr;
    v.k_s = t->dev_pre_spt_s; v.g_s = t->dev_dec_spt_s; v.c = t->dev_ttft_c;
    return v;
}

int check_trace(const disco_trace* t)
{
    if (!t) return DISCO_ERR_NULL;
    if (t->n_req < 0 || t->n_tok < 0) return DISCO_ERR_SHAPE;
    if (t->n_req > 0 && (!t->prompt_len || !t->output_len || !t->srv_ttft)) return DISCO_ERR_NULL;
    if ((t->tok_arr != nullptr) != (t->tok_off != nullptr) && t->tok_arr) return DISCO_ERR_CSR;
    return DISCO_OK;
}

int check_policies(const disco_policy* pol, int P)
{
    if (!pol) return DISCO_ERR_NULL;
    if (P < 1 || P > DISCO_MAX_COLS) return DISCO_ERR_SHAPE;
    for (int j = 0; j < P; ++j) {
        if (pol[j].mode < DISCO_MODE_SERVER_CONSTRAINED || pol[j].mode > DISCO_MODE_STOCH_DEVICE) return DISCO_ERR_RANGE;
        if (pol[j].mode >= DISCO_MODE_STOCH_SERVER && !(pol[j].beta >= 0.0f && pol[j].beta <= 1.0f))
            return DISCO_ERR_RANGE;                         // the routing probability of a stochastic baseline
        if (pol[j].mig_mode != DISCO_MIG_NONE && pol[j].mig_mode != DISCO_MIG_LAG && pol[j].mig_mode != DISCO_MIG_BUFFER)
            return DISCO_ERR_RANGE;
        if (pol[j].w_mid != pol[j].w_mid || pol[j].beta != pol[j].beta || pol[j].w_tail != pol[j].w_tail)
            return DISCO_ERR_RANGE;
    }
    return DISCO_OK;
}

int check_ws(void* ws, size_t ws_bytes, int P)
{
    if (!ws) return DISCO_ERR_WORKSPACE;
    if (ws_bytes < disco_ws_layout(P).total) return DISCO_ERR_WORKSPACE;
    if (((uintptr_t)ws & 255u) != 0) return DISCO_ERR_WORKSPACE;
    return DISCO_OK;
}

// Prices of the buffer hand-off's cost test from the unified cost rates (Sec. 4.1): a server source saves
// cs_dec - lambda e_dec per token and pays lambda e_pre per re-prefilled token; a device source the mirror image.
// Without rates nothing is ever saved (no hand-off).
BufCostArgs buffer_prices(const disco_cost_params* c)
{
    BufCostArgs b{0.0, 0.0, 0.0, 0.0};
    if (c) {
        const double dev_dec = c->lambda * c->e_dec, dev_pre = c->lambda * c->e_pre;
        b.dc_srv = c->cs_dec - dev_dec; b.cp_srv = dev_pre;
        b.dc_dev = dev_dec - c->cs_dec; b.cp_dev = c->cs_pre;
    }
    return b;
}

bool is_device_pointer(const void* p)
{
    hipPointerAttribute_t attr;
    if (hipPointerGetAttributes(&attr, p) != hipSuccess) {
        (void)hipGetLastError();          // ordinary host memory is not known to the runtime
        return false;
    }
    return attr.type == hipMemoryTypeDevice;
}

// Host tables are validated and travel as a kernel argument; device tables
// (e.g. the pol_out of a budget search) are copied on the device, unvalidated.
int stage_policies(const disco_policy* pol, int P, char* ws, const WsLayout& L, hipStream_t stream, const SelInit* sel = nullptr)
{
    SelInit si;
    memset(&si, 0, sizeof(si));
    if (sel) si = *sel;
    if (!pol) return DISCO_ERR_NULL;
    if (P < 1 || P > DISCO_MAX_COLS) return DISCO_ERR_SHAPE;
    if (is_device_pointer(pol)) {
        hipLaunchKernelGGL(k_copy_policies, dim3(1), dim3(STAGE_THREADS), 0, stream, pol, P, (disco_policy*)(ws + L.pol),
                           (unsigned*)(ws + L.ticket), (u64*)(ws + L.part), si);
        return DISCO_OK;
    }
    int rc = check_policies(pol, P);
    if (rc) return rc;
    PolTable t;
    memset(&t, 0, sizeof(t));
    memcpy(t.p, pol, sizeof(disco_policy) * (size_t)P);
    hipLaunchKernelGGL(k_store_policies, dim3(1), dim3(STAGE_THREADS), 0, stream, t, P, (disco_policy*)(ws + L.pol),
                       (unsigned*)(ws + L.ticket), (u64*)(ws + L.part), si);
    return DISCO_OK;
}

}  // namespace

void disco_set_hip_error(hipError_t e, const char* what)
{
    snprintf(g_hip_error, sizeof(g_hip_error), "%s: %s", what, hipGetErrorString(e));
}

WsLayout disco_ws_layout(int32_t P)
{
    auto up = [](size_t x) { return (x + 255) & ~(size_t)255; };
    WsLayout L;
    size_t o = 0;
    L.pol = o; o += up(sizeof(disco_policy) * DISCO_MAX_COLS);
    L.ticket = o; o += up(sizeof(unsigned) * 64);
    L.search = o; o += up(sizeof(SearchState) * DISCO_MAX_COLS);
    L.sel = o; o += up(sizeof(SelState));
    L.ghist = o; o += up(sizeof(unsigned) * DISCO_GHIST_WORDS);
    L.part = o;
    (void)P;
    o += up((size_t)DISCO_MAX_BLOCKS * 64 * 64);     // workgroups x columns x 64-byte partial
    L.ppcnt = o; o += up(sizeof(unsigned) * DISCO_MAX_CLS * (DISCO_PP_NMAX + 1));
    L.dhist = o; o += up(sizeof(unsigned) * DISCO_MAX_COLS * DISCO_DELAY_BINS);
    L.templ = o; o += up(sizeof(disco_policy) * DISCO_MAX_COLS);
    L.wcount = o; o += up(sizeof(unsigned) * 1024);
    L.slices = o; o += up((size_t)256 * (2 * DISCO_MAX_COLS + 2) * 256 * sizeof(unsigned));   // 256 workgroups x rows x bins
    L.total = o;
    return L;
}

// The fixed regions, then one byte and 16 bytes per request (see disco_ws_bytes_region).
extern "C" size_t disco_workspace_bytes(int64_t n_req, int32_t P)
{
    return disco_ws_full_bytes(disco_ws_layout(P), n_req);
}

extern "C" const char* disco_strerror(int32_t code)
{
    switch (code) {
    case DISCO_OK: return "ok";
    case DISCO_ERR_NULL: return "a required pointer is NULL";
    case DISCO_ERR_SHAPE: return "negative or inconsistent sizes";
    case DISCO_ERR_RANGE: return "parameter out of range";
    case DISCO_ERR_CSR: return "token arrays missing or inconsistent";
    case DISCO_ERR_WORKSPACE: return "workspace missing, misaligned or too small";
    case DISCO_ERR_HIP: return "HIP runtime error";
    default: return "unknown error code";
    }
}

extern "C" const char* disco_last_hip_error(void) { return g_hip_error; }

// Alg. 1: the policy type from the unified cost rates (device costs in money = lambda x energy per token).
extern "C" int32_t disco_policy_type(const disco_cost_params* c, int32_t* mode)
{
    if (!c || !mode) return DISCO_ERR_NULL;
    const double cd_p = c->lambda * c->e_pre, cd_d = c->lambda * c->e_dec;
    const double dev_min = cd_p < cd_d ? cd_p : cd_d, srv_max = c->cs_pre > c->cs_dec ? c->cs_pre : c->cs_dec;
    if (dev_min != dev_min || srv_max != srv_max || c->cs_pre != c->cs_pre || c->cs_dec != c->cs_dec) return DISCO_ERR_RANGE;
    *mode = dev_min > srv_max ? DISCO_MODE_DEVICE_CONSTRAINED : DISCO_MODE_SERVER_CONSTRAINED;
    return DISCO_OK;
}

static int g_grid_divisor = 1;
int disco_grid_divisor() { return g_grid_divisor; }
extern "C" int32_t disco_set_grid_divisor(int32_t d)
{
    if (d < 1 || d > 1024) return DISCO_ERR_RANGE;
    g_grid_divisor = d;
    return DISCO_OK;
}
extern "C" int32_t disco_version(void) { return 100; }

extern "C" int32_t disco_eval_dispatch(const disco_trace* trace, const disco_policy* pol, int32_t P,
                                       const disco_pair_out* out, disco_accum* acc, void* ws_, size_t ws_bytes,
                                       void* stream_)
{
    int rc = check_trace(trace);
    if (rc) return rc;
    if (!pol || !acc) return DISCO_ERR_NULL;
    if (P < 1 || P > DISCO_MAX_COLS) return DISCO_ERR_SHAPE;
    rc = check_ws(ws_, ws_bytes, P);
    if (rc) return rc;
    hipStream_t stream = (hipStream_t)stream_;
    char* ws = (char*)ws_;
    const WsLayout L = disco_ws_layout(P);
    const TraceView v = view_of(trace);
    rc = stage_policies(pol, P, ws, L, stream);
    if (rc) return rc;
    DispFin fin;
    memset(&fin, 0, sizeof(fin));
    fin.kind = 0;
    fin.need = 2;
    fin.acc = acc;
    disco_launch_dispatch_acc(v, (const disco_policy*)(ws + L.pol), P, (u64*)(ws + L.part), fin, stream);
    if (out && (out->decision || out->ttft) && v.n_req > 0)
        disco_launch_dispatch_mat(v, (const disco_policy*)(ws + L.pol), P, out->decision, out->ttft, stream);
    DISCO_HIP(hipGetLastError());
    return DISCO_OK;
}

// ---------------------------------------------------- fixed scratch area --
// Scratch of disco_eval_dispatch_static: the three workspace regions a dispatch pass touches (staged policy
// table, flag words, device-wide totals), in device memory that belongs to the library's code object.  Every
// GPU holds its own copy at its own address, which host code obtains once per device from the runtime; the
// array's name is never used as an address on the host.
namespace {
constexpr size_t SS_POL = 0;
constexpr size_t SS_TICKET = SS_POL + sizeof(disco_policy) * DISCO_MAX_COLS;
constexpr size_t SS_PART = SS_TICKET + sizeof(unsigned) * 64;
constexpr size_t SS_TOTALS_BYTES = (size_t)DISCO_NCOPY * 64 * (sizeof(DispPartial) + sizeof(MigPartial));
constexpr size_t SS_BYTES = SS_PART + SS_TOTALS_BYTES;
static_assert(SS_TICKET % 256 == 0 && SS_PART % 256 == 0, "regions of the fixed scratch are 256-byte aligned");
static_assert(SS_BYTES == DISCO_STATIC_SCRATCH_BYTES, "the size the public header states");
}  // namespace

static __device__ __align__(256) unsigned char scratch[SS_BYTES];

namespace {
constexpr int SS_MAX_DEVICES = 64;
std::mutex g_scratch_mutex;
char* g_scratch_ptr[SS_MAX_DEVICES];       // device address of `scratch` on each GPU, looked up on first use

int static_scratch(char** out)
{
    int dev = -1;
    DISCO_HIP(hipGetDevice(&dev));
    if (dev < 0 || dev >= SS_MAX_DEVICES) return DISCO_ERR_RANGE;
    std::lock_guard<std::mutex> lock(g_scratch_mutex);
    if (!g_scratch_ptr[dev]) {
        void* p = nullptr;
        DISCO_HIP(hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)));
        if (!p || ((uintptr_t)p & 255u) != 0) return DISCO_ERR_WORKSPACE;
        g_scratch_ptr[dev] = (char*)p;
    }
    *out = g_scratch_ptr[dev];
    return DISCO_OK;
}
}  // namespace

extern "C" int32_t disco_eval_dispatch_static(const disco_trace* trace, const disco_policy* pol, int32_t P,
                                              const disco_pair_out* out, disco_accum* acc, void* stream_)
{
    int rc = check_trace(trace);
    if (rc) return rc;
    if (!pol || !acc) return DISCO_ERR_NULL;
    if (P < 1 || P > DISCO_MAX_COLS) return DISCO_ERR_SHAPE;       // the scratch holds DISCO_MAX_COLS columns
    char* ws = nullptr;
    rc = static_scratch(&ws);
    if (rc) return rc;
    hipStream_t stream = (hipStream_t)stream_;
    WsLayout L;
    memset(&L, 0, sizeof(L));
    L.pol = SS_POL; L.ticket = SS_TICKET; L.part = SS_PART; L.total = SS_BYTES;
    const TraceView v = view_of(trace);
    rc = stage_policies(pol, P, ws, L, stream);        // also puts the flag words and the totals at their identity
    if (rc) return rc;
    DispFin fin;
    memset(&fin, 0, sizeof(fin));
    fin.kind = 0;
    fin.need = 2;
    fin.acc = acc;
    disco_launch_dispatch_acc(v, (const disco_policy*)(ws + L.pol), P, (u64*)(ws + L.part), fin, stream);
    if (out && (out->decision || out->ttft) && v.n_req > 0)
        disco_launch_dispatch_mat(v, (const disco_policy*)(ws + L.pol), P, out->decision, out->ttft, stream);
    DISCO_HIP(hipGetLastError());
    return DISCO_OK;
}

extern "C" int32_t disco_eval_migration(const disco_trace* trace, const disco_timeline_params* tl,
                                        const disco_policy* pol, int32_t P, const disco_mig_out* out,
                                        disco_accum* acc, void* ws_, size_t ws_bytes, void* stream_)
{
    int rc = check_trace(trace);
    if (rc) return rc;
    if (!tl || !pol || !acc) return DISCO_ERR_NULL;
    if (P < 1 || P > DISCO_MAX_COLS) return DISCO_ERR_SHAPE;
    if (!(tl->tau > 0.0f) || !(tl->kappa_lag >= 0.0f)) return DISCO_ERR_RANGE;
    if (trace->n_req > 0 && !trace->tok_arr && !trace->srv_tbt) return DISCO_ERR_CSR;
    if (out && out->delivered && (!trace->tok_off || out->delivered_col < 0 || out->delivered_col >= P))
        return DISCO_ERR_CSR;
    rc = check_ws(ws_, ws_bytes, P);
    if (rc) return rc;
    hipStream_t stream = (hipStream_t)stream_;
    char* ws = (char*)ws_;
    const WsLayout L = disco_ws_layout(P);
    if (!(out && out->delivered) && ws_bytes < disco_ws_full_bytes(L, trace->n_req)) return DISCO_ERR_WORKSPACE;
    TraceView v = view_of(trace);
    if (out && out->delivered) v.off = trace->tok_off;      // offsets index `delivered` even without tok_arr
    rc = stage_policies(pol, P, ws, L, stream);
    if (rc) return rc;
    TimelineArgs a;
    memset(&a, 0, sizeof(a));
    a.tau = tl->tau;
    a.kt = tl->kappa_lag * tl->tau;
    a.P = P; a.nq = 1; a.pass = -1;
    if (out) {
        a.mig_idx = out->mig_idx; a.n_src_tok = out->n_src_tok; a.t_last = out->t_last;
        a.delivered = out->delivered; a.delivered_col = out->delivered_col;
        a.delay_num = out->delay_num;
    }
    a.bc = buffer_prices(tl->cost);
    a.buffer_flag = (unsigned*)(ws + L.ticket) + DISCO_FLAG_BUFFER;
    a.part = (MigPartial*)(ws + L.part);
    a.ticket = (unsigned*)(ws + L.ticket);
    a.acc = acc;
    a.S = (SelState*)(ws + L.sel);
    a.ghist = (unsigned*)(ws + L.ghist);
    // Streaming kernels (token walk into per-request summaries, per-column totals from them, then the pairs with a
    // buffer hand-off), unless per-token deliveries are wanted: then the general kernel.
    if (a.delivered) {
        disco_launch_timeline_general(v, trace->n_tok, (const disco_policy*)(ws + L.pol), a, stream);
    } else {
        a.wflags = (unsigned char*)(ws + L.total);
        a.summary = ws + disco_ws_summary_offset(L, v.n_req);
        a.counter = (unsigned*)(ws + L.wcount);
        a.bufsum = ws + disco_ws_bufsum_offset(L, v.n_req);
        disco_launch_tl_stats_fast(v, trace->n_tok, (const disco_policy*)(ws + L.pol), a,
                                   tl_totals((u64*)(ws + L.part)), stream);
    }
    DISCO_HIP(hipGetLastError());
    return DISCO_OK;
}

// Measurement aid: the streaming token walk of disco_eval_migration, timed alone with HIP events on `stream`.
extern "C" int32_t disco_time_token_walk(const disco_trace* trace, const disco_timeline_params* tl, const disco_policy* pol,
                                         int32_t P, void* ws_, size_t ws_bytes, int32_t reps, double* mean_ms, double* min_ms,
                                         void* stream_)
{
    int rc = check_trace(trace);
    if (rc) return rc;
    if (!tl || !pol || !mean_ms || !min_ms) return DISCO_ERR_NULL;
    if (P < 1 || P > DISCO_MAX_COLS || reps < 1 || reps > 1000) return DISCO_ERR_SHAPE;
    if (!(tl->tau > 0.0f) || !(tl->kappa_lag >= 0.0f)) return DISCO_ERR_RANGE;
    if (trace->n_req <= 0 || !trace->tok_arr) return DISCO_ERR_CSR;          // the streaming walk reads a token array
    rc = check_ws(ws_, ws_bytes, P);
    if (rc) return rc;
    hipStream_t stream = (hipStream_t)stream_;
    char* ws = (char*)ws_;
    const WsLayout L = disco_ws_layout(P);
    if (ws_bytes < disco_ws_full_bytes(L, trace->n_req)) return DISCO_ERR_WORKSPACE;
    const TraceView v = view_of(trace);
    rc = stage_policies(pol, P, ws, L, stream);
    if (rc) return rc;
    hipEvent_t e0 = nullptr, e1 = nullptr;
    DISCO_HIP(hipEventCreate(&e0));
    DISCO_HIP(hipEventCreate(&e1));
    double sum = 0.0, best = 1e300;
    for (int r = 0; r <= reps && rc == DISCO_OK; ++r) {          // the first run warms up and is not counted
        disco_launch_tl_walk(v, trace->n_tok, (const disco_policy*)(ws + L.pol), P, tl->tau, tl->kappa_lag * tl->tau,
                             (unsigned char*)(ws + L.total), ws + disco_ws_summary_offset(L, v.n_req), (unsigned*)(ws + L.wcount),
                             stream, e0, e1);
        hipError_t e = hipEventSynchronize(e1);
        float ms = 0.0f;
        if (e == hipSuccess) e = hipEventElapsedTime(&ms, e0, e1);
        if (e == hipSuccess) e = hipStreamSynchronize(stream);
        if (e != hipSuccess) { disco_set_hip_error(e, "timing the token walk"); rc = DISCO_ERR_HIP; }
        if (r > 0) { sum += ms; if (ms < best) best = ms; }
    }
    (void)hipEventDestroy(e0);
    (void)hipEventDestroy(e1);
    if (rc) return rc;
    *mean_ms = sum / reps;
    *min_ms = best;
    return DISCO_OK;
}

extern "C" int32_t disco_reduce_stats(const disco_trace* trace, const disco_cost_params* cost,
                                      const disco_timeline_params* tl, const disco_policy* pol, int32_t P,
                                      const disco_accum* acc, const disco_quantile* q, int32_t nq, disco_stats* out,
                                      void* ws_, size_t ws_bytes, void* stream_)
{
    int rc = check_trace(trace);
    if (rc) return rc;
    if (!cost || !acc || !out || !pol) return DISCO_ERR_NULL;
    if (P < 1 || P > DISCO_MAX_COLS) return DISCO_ERR_SHAPE;
    if (nq < 0 || nq > DISCO_MAX_Q || (nq > 0 && !q)) return nq > 0 && !q ? DISCO_ERR_NULL : DISCO_ERR_SHAPE;
    if (P * nq > DISCO_MAX_SLOTS) return DISCO_ERR_SHAPE;
    for (int i = 0; i < nq; ++i)
        if (q[i].den <= 0 || q[i].num < 0 || q[i].num > q[i].den) return DISCO_ERR_RANGE;
    if (tl && (!(tl->tau > 0.0f) || !(tl->kappa_lag >= 0.0f))) return DISCO_ERR_RANGE;
    if (tl && trace->n_req > 0 && !trace->tok_arr && !trace->srv_tbt) return DISCO_ERR_CSR;
    if (tl && nq > 0 && trace->n_req > 0xFFFFFFFFll) return DISCO_ERR_SHAPE;     // the walk list holds 32-bit request indices
    rc = check_ws(ws_, ws_bytes, P);
    if (rc) return rc;
    hipStream_t stream = (hipStream_t)stream_;
    char* ws = (char*)ws_;
    const WsLayout L = disco_ws_layout(P);
    if (tl && nq > 0 && ws_bytes < disco_ws_full_bytes(L, trace->n_req)) return DISCO_ERR_WORKSPACE;
    const TraceView v = view_of(trace);
    SelState* S = (SelState*)(ws + L.sel);
    unsigned* gh = (unsigned*)(ws + L.ghist);
    disco_quantile qs[4] = {{0, 1}, {0, 1}, {0, 1}, {0, 1}};
    for (int i = 0; i < nq; ++i) qs[i] = q[i];
    SelInit si;
    memset(&si, 0, sizeof(si));
    si.S = S; si.nq = nq; si.acc = acc; si.n_req = v.n_req;
    for (int i = 0; i < 4; ++i) si.q[i] = qs[i];
    si.with_tbt = tl != nullptr;
    rc = stage_policies(pol, P, ws, L, stream, nq > 0 ? &si : nullptr);        // with the start of the TTFT selection
    if (rc) return rc;
    if (nq > 0) {
        unsigned char* ubytes = ws_bytes >= L.total + (size_t)v.n_req ? (unsigned char*)(ws + L.total) : nullptr;
        for (int pass = 0; pass < 4; ++pass)
            disco_launch_ttft_pass(v, (const disco_policy*)(ws + L.pol), P, nq, pass, S, (unsigned*)(ws + L.slices), gh,
                                   ubytes, stream);
        if (tl) {
            TimelineArgs a;
            memset(&a, 0, sizeof(a));
            a.tau = tl->tau;
            a.kt = tl->kappa_lag * tl->tau;
            a.P = P; a.nq = nq;
            a.ticket = (unsigned*)(ws + L.ticket);
            a.S = S; a.ghist = gh;
            a.bc = buffer_prices(tl->cost);          // the prices the statistics pass used
            a.dhist = (unsigned*)(ws + L.dhist);
            a.buffer_flag = (unsigned*)(ws + L.ticket) + DISCO_FLAG_BUFFER;
            // column sets -> classes, then the radix passes; the digits are sized on the device and
            // launches after the last needed pass return at once
            a.ppcnt = (unsigned*)(ws + L.ppcnt);
            const disco_policy* dpol = (const disco_policy*)(ws + L.pol);
            // what the token walk found per request: left in the workspace by disco_eval_migration, or walked now
            a.wflags = (unsigned char*)(ws + L.total);
            a.summary = ws + disco_ws_summary_offset(L, v.n_req);
            a.counter = (unsigned*)(ws + L.wcount);
            a.bufsum = ws + disco_ws_bufsum_offset(L, v.n_req);
            if (!tl->reuse_walk) {
                disco_launch_tl_walk(v, trace->n_tok, dpol, P, a.tau, a.kt, a.wflags, a.summary, a.counter, stream);
                disco_launch_tl_stats_buf(v, trace->n_tok, dpol, a, nullptr, stream);      // summaries only
            }
            disco_launch_tl_classify(v, dpol, P, nq, tl->tau, a.summary, a.bufsum, S, a.ppcnt, gh, a.dhist,
                                     (unsigned*)(ws + L.ticket), stream);
            a.desc = (u64*)(ws + disco_ws_desc_offset(L, v.n_req));
            a.list = (unsigned*)(a.desc + v.n_req);
            disco_launch_tl_assign(v, dpol, P, a.summary, S, a.bufsum, a.desc, a.list, (unsigned*)(ws + L.slices),
                                   L.total - L.slices, a.ppcnt, a.dhist, stream);
            disco_launch_pp_suffix(S, a.ppcnt, stream);
            for (int pass = 0; pass < DISCO_TBT_MAX_PASS; ++pass) {
                a.pass = pass;
                if (pass < DISCO_TBT_REGULAR_PASS) disco_launch_tl_hist_fast(v, trace->n_tok, dpol, a, stream);
                disco_launch_tbt_pass(v, trace->n_tok, dpol, a, stream);
            }
        }
    }
    const bool per_column = tl && nq > 0;
    hipLaunchKernelGGL(k_stats_final, dim3(per_column ? (unsigned)P : 1u), dim3(per_column ? 256 : 64), 0, stream, P, nq, v.n_req,
                       *cost, tl ? 1 : 0, acc, S, qs[0], qs[1], qs[2], qs[3], (const unsigned*)(ws + L.dhist), out);
    DISCO_HIP(hipGetLastError());
    return DISCO_OK;
}

extern "C" int32_t disco_average_runs(const disco_stats* in, int32_t groups, int32_t runs, disco_stats* out, void* stream_)
{
    if (!in || !out) return DISCO_ERR_NULL;
    if (groups < 0 || runs < 1) return DISCO_ERR_SHAPE;
    if (groups == 0) return DISCO_OK;
    hipLaunchKernelGGL(k_average_runs, dim3((unsigned)((groups + 63) / 64)), dim3(64), 0, (hipStream_t)stream_, in, groups, runs,
                       out);
    DISCO_HIP(hipGetLastError());
    return DISCO_OK;
}

extern "C" int32_t disco_ingest_trace(const disco_raw_trace* raw, disco_trace* trace, void* stream_)
{
    if (!raw || !trace) return DISCO_ERR_NULL;
    if (raw->n_req < 0 || raw->n_tok < 0) return DISCO_ERR_SHAPE;
    if (raw->n_req > 0 && (!raw->t_send || !raw->tok_off || !trace->srv_ttft || !trace->output_len)) return DISCO_ERR_NULL;
    if (raw->n_tok > 0 && (!raw->t_token || !trace->tok_arr)) return DISCO_ERR_NULL;
    trace->n_req = raw->n_req;
    trace->n_tok = raw->n_tok;
    trace->tok_off = const_cast<int64_t*>(raw->tok_off);
    if (raw->n_req == 0) return DISCO_OK;
    disco_launch_ingest(raw->n_req, raw->t_send, raw->t_token, raw->tok_off, trace->srv_ttft, trace->output_len,
                        trace->tok_arr, (hipStream_t)stream_);
    DISCO_HIP(hipGetLastError());
    return DISCO_OK;
}

extern "C" int32_t disco_fit_lognormal(const void* x, int32_t kind, int64_t n, disco_lognormal_fit* out, void* ws_,
                                       size_t ws_bytes, void* stream_)
{
    if (!out || (n > 0 && !x)) return DISCO_ERR_NULL;
    if (n < 0) return DISCO_ERR_SHAPE;
    if (kind != DISCO_FIT_INT32 && kind != DISCO_FIT_FLOAT32) return DISCO_ERR_RANGE;
    int rc = check_ws(ws_, ws_bytes, 1);
    if (rc) return rc;
    const WsLayout L = disco_ws_layout(1);
    if (disco_fit_scratch_bytes() > L.total - L.slices) return DISCO_ERR_WORKSPACE;
    disco_launch_fit(x, kind, n, out, (char*)ws_ + L.slices, (hipStream_t)stream_);
    DISCO_HIP(hipGetLastError());
    return DISCO_OK;
}

extern "C" int32_t disco_solve_policy(const disco_trace* trace, const disco_solve_spec* spec, int32_t n, disco_policy* pol_out,
                                      disco_solve_out* out, void* ws_, size_t ws_bytes, void* stream_)
{
    int rc = check_trace(trace);
    if (rc) return rc;
    if (!spec || !pol_out) return DISCO_ERR_NULL;
    if (n < 1 || n > DISCO_MAX_COLS) return DISCO_ERR_SHAPE;
    for (int j = 0; j < n; ++j) {
        const disco_solve_spec& s = spec[j];
        if (s.mode != DISCO_MODE_SERVER_CONSTRAINED && s.mode != DISCO_MODE_DEVICE_CONSTRAINED) return DISCO_ERR_RANGE;
        if (s.b_den < 1 || s.b_den > 32768 || s.b_num < 0 || s.b_num > s.b_den) return DISCO_ERR_RANGE;
        if (s.mode == DISCO_MODE_DEVICE_CONSTRAINED &&
            (s.a_den < 1 || s.a_den > 32768 || s.a_num <= 0 || s.a_num >= s.a_den))
            return DISCO_ERR_RANGE;
        if (s.mig_mode < DISCO_MIG_NONE || s.mig_mode > DISCO_MIG_BUFFER) return DISCO_ERR_RANGE;
    }
    rc = check_ws(ws_, ws_bytes, n);
    if (rc) return rc;
    char* ws = (char*)ws_;
    const WsLayout L = disco_ws_layout(n);
    if (disco_solve_state_bytes() > L.ghist - L.sel) return DISCO_ERR_WORKSPACE;      // the selection state region holds it
    const TraceView v = view_of(trace);
    disco_launch_solve(v, spec, n, ws + L.sel, (u64*)(ws + L.ppcnt), (u64*)((unsigned*)(ws + L.ticket) + 32),
                       (unsigned*)(ws + L.slices), L.total - L.slices, pol_out, out, (hipStream_t)stream_);
    DISCO_HIP(hipGetLastError());
    return DISCO_OK;
}

extern "C" int32_t disco_budget_search(const disco_trace* trace, const disco_cost_params* cost,
                                       const disco_policy* templ, const disco_search_spec* spec, int32_t n_search,
                                       disco_search_out* out, disco_policy* pol_out, disco_accum* acc_out, void* ws_,
                                       size_t ws_bytes, void* stream_)
{
    int rc = check_trace(trace);
    if (rc) return rc;
    if (!cost || !spec || !out || !templ) return DISCO_ERR_NULL;
    if (n_search < 1 || n_search > DISCO_MAX_COLS) return DISCO_ERR_SHAPE;
    const int n_steps = spec[0].n_steps;
    if (n_steps < 1 || n_steps > DISCO_MAX_STEPS) return DISCO_ERR_SHAPE;
    SpecTable t;
    memset(&t, 0, sizeof(t));
    for (int j = 0; j < n_search && !is_device_pointer(templ); ++j)           // the stochastic baselines have no searched parameter
        if (templ[j].mode >= DISCO_MODE_STOCH_SERVER) return DISCO_ERR_RANGE;
    for (int j = 0; j < n_search; ++j) {
        if (spec[j].n_steps != n_steps) return DISCO_ERR_SHAPE;
        if (spec[j].which_param < DISCO_PARAM_L_TH || spec[j].which_param > DISCO_PARAM_BETA) return DISCO_ERR_RANGE;
        if (spec[j].which_acc < DISCO_ACC_TOTAL_COST || spec[j].which_acc > DISCO_ACC_DEVICE_PREFILL_TOK)
            return DISCO_ERR_RANGE;
        if (!(spec[j].lo <= spec[j].hi) || spec[j].target != spec[j].target) return DISCO_ERR_RANGE;
        if (spec[j].which_param == DISCO_PARAM_L_TH && (spec[j].lo < -2147483647.0 || spec[j].hi > 2147483647.0))
            return DISCO_ERR_RANGE;
        t.s[j].lo = spec[j].lo; t.s[j].hi = spec[j].hi; t.s[j].target = spec[j].target;
        t.s[j].which_param = spec[j].which_param; t.s[j].which_acc = spec[j].which_acc;
        t.s[j].step = 0; t.s[j].n_steps = n_steps;
    }
    rc = check_ws(ws_, ws_bytes, n_search);
    if (rc) return rc;
    hipStream_t stream = (hipStream_t)stream_;
    char* ws = (char*)ws_;
    const WsLayout L = disco_ws_layout(n_search);
    const TraceView v = view_of(trace);
    rc = stage_policies(templ, n_search, ws, L, stream);
    if (rc) return rc;
    // Length thresholds of server-constrained columns against a prompt-token budget: the accumulator is a
    // function of the threshold alone and is tabulated once (Alg. 3's sorted running totals); all bisection
    // steps then read the table.  Needs a host-resident template table (its modes are inspected here).
    bool tabulated = v.n_req > 0 && !is_device_pointer(templ);
    double max_hi = 0.0;
    for (int j = 0; j < n_search && tabulated; ++j) {
        tabulated = templ[j].mode == DISCO_MODE_SERVER_CONSTRAINED && spec[j].which_param == DISCO_PARAM_L_TH &&
                    (spec[j].which_acc == DISCO_ACC_SERVER_PREFILL_TOK || spec[j].which_acc == DISCO_ACC_DEVICE_PREFILL_TOK) &&
                    spec[j].lo >= 0.0 && spec[j].hi + 2.0 <= (double)disco_search_table_max_bins();
        if (spec[j].hi > max_hi) max_hi = spec[j].hi;
    }
    // Otherwise every pass evaluates the next `depth` levels of each search's bisection tree as columns of their
    // own and so takes `depth` bisection steps; the recorded steps are those of the plain bisection.
    const int depth = tabulated ? 0 : disco_search_depth(n_search);
    hipLaunchKernelGGL(k_search_init, dim3(1), dim3(64), 0, stream, t, n_search, (SearchState*)(ws + L.search),
                       (disco_policy*)(ws + L.pol), (disco_policy*)(ws + L.templ), depth);
    DispFin fin;
    memset(&fin, 0, sizeof(fin));
    fin.kind = 1;
    fin.cost = *cost;
    fin.st = (SearchState*)(ws + L.search);
    fin.sout = out;
    fin.pol_out = pol_out;
    fin.acc = acc_out;
    fin.pol_rw = (disco_policy*)(ws + L.pol);
    fin.templ = (const disco_policy*)(ws + L.templ);
    fin.n_search = n_search;
    if (tabulated) {
        disco_launch_search_table(v, n_search, (int)max_hi + 2, (unsigned*)(ws + L.slices), L.total - L.slices,
                                  (u64*)(ws + L.ppcnt), (u64*)((unsigned*)(ws + L.ticket) + 32),
                                  (SearchState*)(ws + L.search), (disco_policy*)(ws + L.pol), out, stream);
    } else {
        // bisection passes only need the totals their accumulators are made of
        int need = 0;
        for (int j = 0; j < n_search; ++j)
            if (spec[j].which_acc != DISCO_ACC_SERVER_PREFILL_TOK && spec[j].which_acc != DISCO_ACC_DEVICE_PREFILL_TOK) need = 1;
        const int npass = (n_steps + depth - 1) / depth;
        fin.depth = depth;
        fin.need = need;
        for (int pass = 0; pass < npass; ++pass) {
            fin.last = pass == npass - 1;
            disco_launch_dispatch_acc(v, (const disco_policy*)(ws + L.pol), n_search * ((1 << depth) - 1), (u64*)(ws + L.part),
                                      fin, stream);
        }
    }
    // the evaluation at the answers
    fin.depth = 0; fin.last = 0; fin.need = 2;
    disco_launch_dispatch_acc(v, (const disco_policy*)(ws + L.pol), n_search, (u64*)(ws + L.part), fin, stream);
    DISCO_HIP(hipGetLastError());
    return DISCO_OK;
}
