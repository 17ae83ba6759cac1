// Dispatch passes (Sec. 4.2, Alg. 2 and 3): fused dispatch + per-column
// reduction, the tabulated threshold search of Alg. 3 columns, and the
// materialised per-pair outputs.
//
// Work decomposition: a wave holds up to 64 policy columns in its lanes
// (lane = sub * G + column, G = columns rounded up to a power of two, 64 / G
// request sub-groups) and walks the requests in batches of 64.  A batch is
// loaded coalesced, one request per lane and one batch ahead, staged in LDS,
// and every column lane reads the request of its sub-group with broadcast LDS
// loads.  With a single column (G = 1) lane = request and four consecutive
// requests are fetched per lane with 16-byte loads.  Per-column totals stay
// in registers (32-bit inside a batch, 64-bit across batches) until the end
// of the kernel, are folded over the workgroup and added into a few copies
// of the device-wide totals; a one-workgroup kernel behind the pass
// (k_dispatch_fin) folds the copies in a fixed order and, for a budget
// search, advances the bisection on the device.
#include <math.h>
#include <string.h>

#include <type_traits>

#include "disco_launch.h"
#include "disco_pair.h"
#include "disco_state.h"

namespace {


struct ColTotals {
    u64 s_pre, d_pre, d_dec, started, won;
    double ttft_sum;
    unsigned minb, maxb;
};

__device__ __forceinline__ double acc_value(int which, const disco_cost_params& c, i64 s_pre, i64 s_dec, i64 d_pre,
                                            i64 d_dec)
{
    switch (which) {
    case DISCO_ACC_TOTAL_COST: {
        double server = server_cost_of(c, s_pre, s_dec);
        double energy = device_energy_of(c, d_pre, d_dec);
        double priced = c.lambda * energy;
        return server + priced;
    }
    case DISCO_ACC_SERVER_COST: return server_cost_of(c, s_pre, s_dec);
    case DISCO_ACC_DEVICE_COST: {
        double energy = device_energy_of(c, d_pre, d_dec);
        return c.lambda * energy;
    }
    case DISCO_ACC_SERVER_PREFILL_TOK: return (double)s_pre;
    default: return (double)d_pre;
    }
}

// One bisection step of a search: record (parameter, accumulator), halve the
// bracket, set the parameter of the next evaluation (after the last step: the
// feasible end of the bracket).
__device__ __forceinline__ void search_step(SearchState& st, disco_policy& p, double A, disco_search_out* o)
{
    const int prm = st.which_param;
    const double mid = search_param(prm, p);
    o->hist_param[st.step] = mid;
    o->hist_acc[st.step] = A;
    search_halve(prm, st.lo, st.hi, mid, A > st.target);
    st.step += 1;
    if (st.step < st.n_steps) search_set_mid(prm, st.lo, st.hi, p);
    else search_set_answer(prm, st.hi, p);
}

// Final evaluation of search `col` (Sec. 4.2: the threshold / wait that meets the constrained endpoint's
// budget), at the answer of its bisection.
__device__ void search_finish(int col, const DispFin& fin, const disco_accum& tot)
{
    const SearchState st = fin.st[col];
    const disco_policy p = fin.pol_rw[col];
    const double A = acc_value(st.which_acc, fin.cost, tot.s_pre, tot.s_dec, tot.d_pre, tot.d_dec);
    disco_search_out* o = &fin.sout[col];
    o->param = st.hi;
    o->acc_at_param = A;
    o->lo = st.lo;
    o->hi = st.hi;
    o->at_param = tot;
    if (fin.pol_out) fin.pol_out[col] = p;
    if (fin.acc) {                                  // the evaluation at the answer, as disco_eval_dispatch would leave it
        disco_accum* a = &fin.acc[col];
        a->s_pre = tot.s_pre; a->s_dec = tot.s_dec; a->d_pre = tot.d_pre; a->d_dec = tot.d_dec;
        a->n_dev_started = tot.n_dev_started; a->n_dev_win = tot.n_dev_win; a->ttft_sum = tot.ttft_sum;
        a->ttft_min_bits = tot.ttft_min_bits; a->ttft_max_bits = tot.ttft_max_bits;
    }
}

// A bisection pass has evaluated the next `depth` levels of search j's bisection tree (columns j * M + node - 1
// in heap order, M = 2^depth - 1; folded totals in LDS, word f of column c at sh[f * 64 + c]): walk down the
// tree, one recorded step per level, then write the candidates of the next pass (or, after the last bisection
// pass, the answers).  Called by all threads of the workgroup.
__device__ void search_walk(const DispFin& fin, const u64* sh)
{
    const int j = threadIdx.x, M = (1 << fin.depth) - 1;
    SearchState st;
    if (j < fin.n_search) {
        st = fin.st[j];
        const int prm = st.which_param;
        disco_search_out* o = &fin.sout[j];
        int node = 1;
        for (int d = 0; d < fin.depth && st.step < st.n_steps; ++d) {
            const int c = j * M + node - 1;
            const u64 s_pre = sh[0 * 64 + c], d_pre = sh[1 * 64 + c], d_dec = sh[2 * 64 + c], n_tot = sh[3 * 64 + c];
            const double A = acc_value(st.which_acc, fin.cost, (i64)s_pre, (i64)(n_tot - d_dec), (i64)d_pre, (i64)d_dec);
            const double mid = search_param(prm, fin.pol_rw[c]);
            o->hist_param[st.step] = mid;
            o->hist_acc[st.step] = A;
            const bool above = A > st.target;
            search_halve(prm, st.lo, st.hi, mid, above);
            st.step += 1;
            node = 2 * node + (above ? 1 : 0);
        }
        fin.st[j] = st;
    }
    __syncthreads();                                // every search has read the parameters of its candidates
    if (j < fin.n_search) {
        const disco_policy templ = fin.templ[j];
        if (fin.last) {
            disco_policy p = templ;
            search_set_answer(st.which_param, st.hi, p);
            fin.pol_rw[j] = p;
        } else {
            search_write_candidates(st, templ, &fin.pol_rw[j * M], fin.depth);
        }
    }
}

// Device-wide totals of the dispatch passes: 8 words per column (the fields
// of DispPartial), kept word-major in DISCO_NCOPY copies: word f of column c
// in copy k sits at tot[(f * DISCO_NCOPY + k) * 64 + c], so the 64 columns of
// one word are contiguous and a wave reads or updates them with one coalesced
// instruction.  Word 7 holds the smallest TTFT bit pattern in its low half and
// the largest in its high half.
__device__ __forceinline__ u64 fold_word(int f, u64 a, u64 b)
{
    if (f < 6) return a + b;
    if (f == 6) return (u64)__double_as_longlong(__longlong_as_double((long long)a) + __longlong_as_double((long long)b));
    const unsigned lo = min((unsigned)a, (unsigned)b), hi = max((unsigned)(a >> 32), (unsigned)(b >> 32));
    return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ bool word_needed(int f, int need) { return f < 2 || (need >= 1 && f < 6) || need >= 2; }

// Workgroup totals -> device-wide totals.  The per-wave partials are in LDS
// (word f of partial r at sh[f * DP_BLOCK + r], rows = waves x G columns);
// wave f folds word f over the waves and adds it into one of the copies with
// one atomic instruction (exact integer atomics; the fp64 TTFT sum is
// order-dependent in its last bits).
template <int G>
__device__ __forceinline__ void add_to_totals(const u64* sh, u64* tot, int P, int need)
{
    const int f = threadIdx.x >> 6, c = threadIdx.x & 63;
    if (f >= 8 || c >= G || !word_needed(f, need)) return;
    u64 x = sh[f * DP_BLOCK + c];
#pragma unroll
    for (int w = 1; w < DP_WAVES; ++w) x = fold_word(f, x, sh[f * DP_BLOCK + w * G + c]);
    if (c >= P) return;
    u64* dst = &tot[(f * DISCO_NCOPY + (int)(blockIdx.x % DISCO_NCOPY)) * 64 + c];
    if (f < 6) atomicAdd((unsigned long long*)dst, (unsigned long long)x);
    else if (f == 6) unsafeAtomicAdd(reinterpret_cast<double*>(dst), __longlong_as_double((long long)x));   // hardware fp64 add (the workspace is ordinary device memory)
    else {
        atomicMin(reinterpret_cast<unsigned*>(dst), (unsigned)x);
        atomicMax(reinterpret_cast<unsigned*>(dst) + 1, (unsigned)(x >> 32));
    }
}

// After the pass (k_dispatch_fin): wave f reads the copies of word f, puts them back to their
// identity for the next pass and folds them in order; then thread = column
// hands the sums to the accumulator or to the search.
__device__ __forceinline__ void finish_columns(u64* tot, int P, const DispFin& fin, u64* sh /* LDS */)
{
    const int f = threadIdx.x >> 6, c = threadIdx.x & 63;
    if (f < 8 && c < P) {
        u64 v[DISCO_NCOPY];
#pragma unroll
        for (int k = 0; k < DISCO_NCOPY; ++k)
            v[k] = __hip_atomic_load(&tot[(f * DISCO_NCOPY + k) * 64 + c], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        const u64 identity = f == 7 ? 0x00000000FFFFFFFFull : 0ull;
#pragma unroll
        for (int k = 0; k < DISCO_NCOPY; ++k) tot[(f * DISCO_NCOPY + k) * 64 + c] = identity;
        u64 x = v[0];
#pragma unroll
        for (int k = 1; k < DISCO_NCOPY; ++k) x = fold_word(f, x, v[k]);
        sh[f * 64 + c] = x;
    }
    __syncthreads();
    if (fin.kind == 1 && fin.depth > 0) {
        search_walk(fin, sh);
        return;
    }
    if ((int)threadIdx.x < P) {
        const int c = threadIdx.x;
        const u64 n_tot = sh[3 * 64 + c], d_dec = sh[2 * 64 + c];
        disco_accum acc;
        memset(&acc, 0, sizeof(acc));
        acc.s_pre = (i64)sh[0 * 64 + c]; acc.d_pre = (i64)sh[1 * 64 + c]; acc.d_dec = (i64)d_dec;
        acc.s_dec = (i64)(n_tot - d_dec);
        acc.n_dev_started = (i64)sh[4 * 64 + c]; acc.n_dev_win = (i64)sh[5 * 64 + c];
        acc.ttft_sum = __longlong_as_double((long long)sh[6 * 64 + c]);
        acc.ttft_min_bits = (unsigned)sh[7 * 64 + c]; acc.ttft_max_bits = (unsigned)(sh[7 * 64 + c] >> 32);
        if (fin.kind == 0) {
            disco_accum* o = &fin.acc[c];
            o->s_pre = acc.s_pre; o->s_dec = acc.s_dec; o->d_pre = acc.d_pre; o->d_dec = acc.d_dec;
            o->n_dev_started = acc.n_dev_started; o->n_dev_win = acc.n_dev_win; o->ttft_sum = acc.ttft_sum;
            o->ttft_min_bits = acc.ttft_min_bits; o->ttft_max_bits = acc.ttft_max_bits;
        } else {
            search_finish(c, fin, acc);
        }
    }
}

// ------------------------------------------------- fused dispatch + reduce --


// Inner loop over the G requests of this lane's sub-group.
// NEED 0: prefill token totals only; 1: + decode split and winner counts;
// 2: + TTFT sum and range (a budget search needs less than an evaluation).
// Fast form: full batch (no validity masks; lanes of unused columns compute
// garbage nobody reads) and every l, n of the batch below 2^24, so the batch
// totals fit 32-bit registers.
template <int G, int MODE, int NEED, bool RAGGED>
__device__ __forceinline__ void batch_pairs_fast(const Staged* __restrict__ st, int sub, int cnt, i64 base, const disco_policy& p,
                                                 ColTotals& t, const StochRuns& runs, const float* su)
{
    unsigned sp = 0, dp = 0, dd = 0, ns = 0, nw = 0;
    double ts = 0.0;
    unsigned mn = t.minb, mx = t.maxb;
    // (the mixed form holds wave shuffles, which the compiler does not unroll partially)
    constexpr int UNROLL = MODE == 2 ? 1 : 8;
#pragma unroll UNROLL
    for (int it = 0; it < G; ++it) {
        const Staged r = st[sub * G + it];
        const bool shared = MODE == 2 && runs.on;         // the variate of a stochastic column comes from the batch's draws
        const float u = shared ? stoch_fetch<G == 64>(runs, su, sub * G + it) : 0.0f;
        PairResult e = pair_eval<MODE>(p, r.l, r.s, r.d, base + sub * G + it, shared, u);
        if (RAGGED) {                                  // requests past the end of the trace count for nothing
            const bool v = sub * G + it < cnt;
            e.srv_started = e.srv_started && v; e.dev_started = e.dev_started && v; e.dev_win = e.dev_win && v;
            if (NEED >= 2 && !v) continue;
        }
        if (MODE != 1) sp += e.srv_started ? (unsigned)r.l : 0u;
        if (MODE != 0) dp += e.dev_started ? (unsigned)r.l : 0u;
        if (NEED >= 1) {
            if (MODE != 0) ns += e.dev_started ? 1u : 0u;
            dd += e.dev_win ? (unsigned)r.n : 0u;
            nw += e.dev_win ? 1u : 0u;
        }
        if (NEED >= 2) {
            const unsigned tb = f2u(e.ttft);
            ts += (double)e.ttft;
            mn = min(mn, tb); mx = max(mx, tb);
        }
    }
    t.s_pre += sp; t.d_pre += dp; t.d_dec += dd; t.started += ns; t.won += nw;
    t.ttft_sum += ts;
    t.minb = mn; t.maxb = mx;
}

// Threshold columns (Alg. 3) on a full batch with all l below 2^24 and all n below 2^16: per pair one
// comparison l < l_th and selections between the request's device-only values and its race values, which the
// loading lane has staged.  The selections are written with a bit mask (all ones iff l < l_th): written as
// conditionals the compiler selects between the LDS addresses of the two candidates and loads afterwards, a
// second, dependent trip to LDS per pair.
template <int G, int NEED>
__device__ __forceinline__ void batch_pairs_threshold(const StagedRace* __restrict__ sr, const unsigned* __restrict__ pnr, int sub,
                                                      const disco_policy& p, ColTotals& t)
{
    const unsigned th = (unsigned)(p.l_th < 0 ? 0 : (p.l_th > (1 << 24) ? (1 << 24) : p.l_th));   // same outcome for l < 2^24
    unsigned sp = 0, pk = 0;
    double ts = 0.0;
    unsigned mn = t.minb, mx = t.maxb;
#pragma unroll 8
    for (int it = 0; it < G; ++it) {
        const StagedRace x = sr[sub * G + it];
        const unsigned dev_only = (unsigned)((int)((unsigned)x.l - th) >> 31);     // strict: Alg. 3
        sp += (unsigned)x.l & ~dev_only;
        if (NEED >= 1) pk += (x.pn & dev_only) | (pnr[sub * G + it] & ~dev_only);
        if (NEED >= 2) {
            const unsigned tb = (x.d & dev_only) | (x.m & ~dev_only);
            ts += (double)u2f(tb);
            mn = min(mn, tb); mx = max(mx, tb);
        }
    }
    t.s_pre += sp;
    t.d_dec += pk & ((1u << PN_COUNT_SHIFT) - 1u); t.won += pk >> PN_COUNT_SHIFT;
    t.ttft_sum += ts;
    t.minb = mn; t.maxb = mx;
}

// General form: ragged last batch or huge lengths; everything in 64 bit, every update masked.
template <int G>
__device__ __forceinline__ void batch_pairs_slow(const Staged* __restrict__ st, int sub, int cnt, i64 base, const disco_policy& p,
                                                 bool colv, int mode, ColTotals& t)
{
    for (int it = 0; it < G; ++it) {
        const int src = sub * G + it;
        const Staged r = st[src];
        const PairResult e = pair_eval<2>(p, r.l, r.s, r.d, base + src);
        const bool v = colv && src < cnt;
        if (mode != 1) t.s_pre += (v && e.srv_started) ? (u64)r.l : 0ull;
        if (mode != 0) { t.d_pre += (v && e.dev_started) ? (u64)r.l : 0ull; t.started += (v && e.dev_started) ? 1ull : 0ull; }
        t.d_dec += (v && e.dev_win) ? (u64)r.n : 0ull;
        t.won += (v && e.dev_win) ? 1ull : 0ull;
        t.ttft_sum += v ? (double)e.ttft : 0.0;
        const unsigned tb = f2u(e.ttft);
        t.minb = v ? min(t.minb, tb) : t.minb;
        t.maxb = v ? max(t.maxb, tb) : t.maxb;
    }
}

template <int G, int MODE>
__device__ __forceinline__ void batch_pairs_need(const Staged* __restrict__ st, int sub, int cnt, i64 base, const disco_policy& p,
                                                 int need, ColTotals& t, const StochRuns& runs, const float* su)
{
    if (cnt == 64) {
        if (need == 0) batch_pairs_fast<G, MODE, 0, false>(st, sub, cnt, base, p, t, runs, su);
        else if (need == 1) batch_pairs_fast<G, MODE, 1, false>(st, sub, cnt, base, p, t, runs, su);
        else batch_pairs_fast<G, MODE, 2, false>(st, sub, cnt, base, p, t, runs, su);
    } else {
        batch_pairs_fast<G, MODE, 2, true>(st, sub, cnt, base, p, t, runs, su);
    }
}

template <int G>
__global__ __launch_bounds__(DP_BLOCK) void k_dispatch_acc(TraceView tr, const disco_policy* __restrict__ pol, int P,
                                                           u64* __restrict__ part, DispFin fin)
{
    __shared__ __align__(16) unsigned char smem[DP_BLOCK * sizeof(DispPartial)];    // 64 KB: staging, then folds
    Staged* stage = reinterpret_cast<Staged*>(smem);
    u64* sh = reinterpret_cast<u64*>(smem);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & (G - 1), sub = lane / G;
    const bool colv = col < P;
    const disco_policy p = pol[colv ? col : 0];
    ColTotals t{0, 0, 0, 0, 0, 0.0, 0xFFFFFFFFu, 0u};
    u64 tot_l = 0, tot_n = 0, tot_c = 0;      // column-independent sums, kept by the loading lane
    Staged* st = stage + wave * 64;
    StagedRace* sr = reinterpret_cast<StagedRace*>(smem + DP_BLOCK * sizeof(Staged)) + wave * 64;
    unsigned* pnr = reinterpret_cast<unsigned*>(smem + DP_BLOCK * (sizeof(Staged) + sizeof(StagedRace))) + wave * 64;
    const i64 nbatch = (tr.n_req + 63) >> 6;
    const i64 bstride = (i64)gridDim.x * DP_WAVES;
    // one batch ahead: the loads of the next batch (at first: of the first one, together with the policy
    // record) are in flight while the current one is evaluated
    int lv_n = 0, nv_n = 0;
    float sv_n = 0.0f, kv_n = tr.k_s;
    auto load_batch = [&](i64 b) {
        const i64 i = b * 64 + lane;
        const bool v = b < nbatch && i < tr.n_req;
        lv_n = v ? tr.l[i] : 0;
        nv_n = v ? tr.n[i] : 0;
        sv_n = v ? tr.s[i] : 0.0f;
        kv_n = tr.k ? (v ? tr.k[i] : 0.0f) : tr.k_s;
    };
    i64 b = (i64)blockIdx.x * DP_WAVES + wave;
    load_batch(b);
    const int mode = table_mode(p, colv);
    for (; b < nbatch; b += bstride) {
        const bool v = b * 64 + lane < tr.n_req;
        const int lv = lv_n, nv = nv_n;
        const float sv = sv_n, kv = kv_n;
        load_batch(b + bstride);
        const float dv = __fmaf_rn((float)lv, kv, tr.c);          // device TTFT T_d(l) = k l + c
        tot_l += (u64)lv; tot_n += (u64)nv; tot_c += v ? 1ull : 0ull;
        const int cnt = (int)((tr.n_req - b * 64 < 64) ? (tr.n_req - b * 64) : 64);
        const bool small = __ballot(((unsigned)lv | (unsigned)nv) >= (1u << 24)) == 0ull;
        const bool threshold_form = mode == 0 && cnt == 64 && __ballot((unsigned)lv >= (1u << 24) || (unsigned)nv >= (1u << 16)) == 0ull;
        if (threshold_form) {
            const bool race_dev = dv < sv;                       // ties go to the server
            const unsigned pn = (unsigned)nv | (1u << PN_COUNT_SHIFT);
            sr[lane] = StagedRace{lv, f2u(dv), f2u(race_dev ? dv : sv), pn};
            pnr[lane] = race_dev ? pn : 0u;
        } else {
            st[lane] = Staged{lv, sv, nv, dv};
        }
        // the staging area is private to the wave: no workgroup barrier needed
        __builtin_amdgcn_wave_barrier();
        if (threshold_form) {
            if (fin.need == 0) batch_pairs_threshold<G, 0>(sr, pnr, sub, p, t);
            else if (fin.need == 1) batch_pairs_threshold<G, 1>(sr, pnr, sub, p, t);
            else batch_pairs_threshold<G, 2>(sr, pnr, sub, p, t);
        } else if (small) {
            const StochRuns none{0, -1, 0, false};
            if (mode == 0) batch_pairs_need<G, 0>(st, sub, cnt, b * 64, p, fin.need, t, none, nullptr);
            else if (mode == 1) batch_pairs_need<G, 1>(st, sub, cnt, b * 64, p, fin.need, t, none, nullptr);
            else {
                // (the runs of the table are worked out per batch: kept across the loop they cost the other
                // forms scalar registers)
                const StochRuns runs = stoch_runs(p, colv, lane);
                float su[STOCH_SHARE] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
                if (runs.on) stoch_draw(runs, b * 64 + lane, su);       // this lane's request, every run of the table
                batch_pairs_need<G, 2>(st, sub, cnt, b * 64, p, fin.need, t, runs, su);
            }
        } else {
            batch_pairs_slow<G>(st, sub, cnt, b * 64, p, colv, mode, t);
        }
        __builtin_amdgcn_wave_barrier();
    }
    // column-independent sums: fold over the wave
    tot_l = wave_sum_u64(tot_l); tot_n = wave_sum_u64(tot_n); tot_c = wave_sum_u64(tot_c);
    // fold the request sub-groups of the wave
#pragma unroll
    for (int m = G; m < 64; m <<= 1) {
        t.s_pre += shfl_xor_u64(t.s_pre, m); t.d_pre += shfl_xor_u64(t.d_pre, m); t.d_dec += shfl_xor_u64(t.d_dec, m);
        t.started += shfl_xor_u64(t.started, m); t.won += shfl_xor_u64(t.won, m);
        t.ttft_sum += shfl_xor_f64(t.ttft_sum, m);
        t.minb = min(t.minb, (unsigned)__shfl_xor((int)t.minb, m, 64));
        t.maxb = max(t.maxb, (unsigned)__shfl_xor((int)t.maxb, m, 64));
    }
    // a column that never skips an endpoint charges it every prompt; the device is always started in Alg. 3
    if (mode == 0) { t.d_pre = tot_l; t.started = tot_c; }
    if (mode == 1) t.s_pre = tot_l;
    __syncthreads();                          // staging no longer needed: reuse the LDS for the folds
    if (sub == 0)
        lds_put(sh, DP_BLOCK, wave * G + col,
                DispPartial{t.s_pre, t.d_pre, t.d_dec, tot_n, t.started, t.won, t.ttft_sum, t.minb, t.maxb});
    __syncthreads();
    add_to_totals<G>(sh, part, P, fin.need);
}

// Single column: lane = request, four consecutive requests per lane and
// iteration (16-byte loads when VEC, i.e. all arrays 16-byte aligned).
template <bool VEC>
__global__ __launch_bounds__(DP_BLOCK) void k_dispatch_acc1(TraceView tr, const disco_policy* __restrict__ pol,
                                                            u64* __restrict__ part, DispFin fin)
{
    __shared__ __align__(16) unsigned char smem[DP_BLOCK * sizeof(DispPartial)];
    u64* sh = reinterpret_cast<u64*>(smem);
    const disco_policy p = pol[0];
    const int mode = p.mode == DISCO_MODE_SERVER_CONSTRAINED ? 0 : (p.mode == DISCO_MODE_DEVICE_CONSTRAINED ? 1 : 2);
    ColTotals t{0, 0, 0, 0, 0, 0.0, 0xFFFFFFFFu, 0u};
    u64 tot_n = 0;
    const i64 ngroups = (tr.n_req + 3) >> 2;
    const i64 stride = (i64)gridDim.x * DP_BLOCK;
    for (i64 g4 = (i64)blockIdx.x * DP_BLOCK + threadIdx.x; g4 < ngroups; g4 += stride) {
        int l[4], n[4];
        float s[4], k[4];
        const i64 i0 = g4 * 4;
        if (VEC && i0 + 3 < tr.n_req) {
            const int4 lv = *reinterpret_cast<const int4*>(tr.l + i0);
            const int4 nv = *reinterpret_cast<const int4*>(tr.n + i0);
            const float4 sv = *reinterpret_cast<const float4*>(tr.s + i0);
            l[0] = lv.x; l[1] = lv.y; l[2] = lv.z; l[3] = lv.w;
            n[0] = nv.x; n[1] = nv.y; n[2] = nv.z; n[3] = nv.w;
            s[0] = sv.x; s[1] = sv.y; s[2] = sv.z; s[3] = sv.w;
            if (tr.k) {
                const float4 kv = *reinterpret_cast<const float4*>(tr.k + i0);
                k[0] = kv.x; k[1] = kv.y; k[2] = kv.z; k[3] = kv.w;
            } else { k[0] = k[1] = k[2] = k[3] = tr.k_s; }
        } else {
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const bool v = i0 + q < tr.n_req;
                l[q] = v ? tr.l[i0 + q] : 0; n[q] = v ? tr.n[i0 + q] : 0; s[q] = v ? tr.s[i0 + q] : 0.0f;
                k[q] = tr.k ? (v ? tr.k[i0 + q] : 0.0f) : tr.k_s;
            }
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const bool v = i0 + q < tr.n_req;
            const float d = __fmaf_rn((float)l[q], k[q], tr.c);
            const PairResult e = (mode == 0) ? pair_eval<0>(p, l[q], s[q], d, i0 + q)
                                             : (mode == 1 ? pair_eval<1>(p, l[q], s[q], d, i0 + q) : pair_eval<2>(p, l[q], s[q], d, i0 + q));
            t.s_pre += (v && e.srv_started) ? (u64)l[q] : 0ull;
            t.d_pre += (v && e.dev_started) ? (u64)l[q] : 0ull;
            if (fin.need >= 1) {
                t.started += (v && e.dev_started) ? 1ull : 0ull;
                t.d_dec += (v && e.dev_win) ? (u64)n[q] : 0ull;
                t.won += (v && e.dev_win) ? 1ull : 0ull;
                tot_n += v ? (u64)n[q] : 0ull;
            }
            if (fin.need >= 2) {
                t.ttft_sum += v ? (double)e.ttft : 0.0;
                const unsigned tb = f2u(e.ttft);
                t.minb = v ? min(t.minb, tb) : t.minb;
                t.maxb = v ? max(t.maxb, tb) : t.maxb;
            }
        }
    }
    t.s_pre = wave_sum_u64(t.s_pre); t.d_pre = wave_sum_u64(t.d_pre);
    if (fin.need >= 1) {
        t.d_dec = wave_sum_u64(t.d_dec); t.started = wave_sum_u64(t.started); t.won = wave_sum_u64(t.won);
        tot_n = wave_sum_u64(tot_n);
    }
    if (fin.need >= 2) {
        t.ttft_sum = wave_sum_f64(t.ttft_sum);
        t.minb = wave_min_u32(t.minb); t.maxb = wave_max_u32(t.maxb);
    }
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    if (lane == 0)
        lds_put(sh, DP_BLOCK, wave, DispPartial{t.s_pre, t.d_pre, t.d_dec, tot_n, t.started, t.won, t.ttft_sum, t.minb, t.maxb});
    __syncthreads();
    add_to_totals<1>(sh, part, 1, fin.need);
}

// Device-wide totals -> accumulators or search steps (one workgroup, launched behind a dispatch pass: a kernel
// boundary costs less than a ticket chain at the end of the pass).
__global__ __launch_bounds__(512) void k_dispatch_fin(u64* __restrict__ part, int P, DispFin fin)
{
    __shared__ u64 sh[8 * 64];
    finish_columns(part, P, fin, sh);
}

// Materialised per-pair outputs, lane = request so that every column is
// written coalesced.
__global__ __launch_bounds__(256) void k_dispatch_mat(TraceView tr, const disco_policy* __restrict__ pol, int P,
                                                      uint8_t* __restrict__ decision, float* __restrict__ ttft)
{
    __shared__ disco_policy sp[DISCO_MAX_COLS];
    if ((int)threadIdx.x < P) sp[threadIdx.x] = pol[threadIdx.x];
    __syncthreads();
    for (i64 i = (i64)blockIdx.x * blockDim.x + threadIdx.x; i < tr.n_req; i += (i64)gridDim.x * blockDim.x) {
        const int l = tr.l[i];
        const float s = tr.s[i];
        const float k = tr.k ? tr.k[i] : tr.k_s;
        const float d = __fmaf_rn((float)l, k, tr.c);
        for (int j = 0; j < P; ++j) {
            unsigned dec; float t;
            dispatch_pair(sp[j], l, s, d, i, dec, t);
            if (decision) decision[(size_t)j * tr.n_req + i] = (uint8_t)dec;
            if (ttft) ttft[(size_t)j * tr.n_req + i] = t;
        }
    }
}

// ---------------------------------------------- threshold search, Alg. 3 ----
//
// Server-constrained columns (Alg. 3): the server's share of the prompt tokens
// is A(L) = sum of l_i over requests with l_i >= L, a function of the length
// threshold alone.  As in Alg. 3 (lengths in order, running totals) the whole
// function is tabulated once -- requests per prompt length, then suffix sums
// of count x length -- and every bisection step of every column reads the
// table instead of passing over the requests.  The steps, their order and the
// recorded history are those of the generic search.

constexpr int LH_MAX_BINS = 32772;          // 128 KB of LDS counts: prompt lengths 0 .. 32771

// Requests per prompt length, one slice of `nbins` counts per workgroup; the
// lengths of requests outside [0, nbins) are added up in `other`.
__global__ __launch_bounds__(DP_BLOCK) void k_len_hist(TraceView tr, int nbins, unsigned* __restrict__ slices, u64* other)
{
    __shared__ unsigned cnt[LH_MAX_BINS];
    for (int i = threadIdx.x; i < nbins; i += DP_BLOCK) cnt[i] = 0u;
    __syncthreads();
    u64 out = 0;
    for (i64 i = (i64)blockIdx.x * DP_BLOCK + threadIdx.x; i < tr.n_req; i += (i64)gridDim.x * DP_BLOCK) {
        const int l = tr.l[i];
        if (l >= 0 && l < nbins) atomicAdd(&cnt[l], 1u);
        else if (l > 0) out += (u64)l;
    }
    out = wave_sum_u64(out);
    if ((threadIdx.x & 63) == 0 && out) atomicAdd((unsigned long long*)other, (unsigned long long)out);
    __syncthreads();
    unsigned* mine = slices + (size_t)blockIdx.x * nbins;
    for (int i = threadIdx.x; i < nbins; i += DP_BLOCK) mine[i] = cnt[i];
}

// table[v] = v x (requests of length v), summed over the slices: 64 lengths
// per workgroup, each of the 16 waves takes every sixteenth slice with four
// loads in flight (the pass is a chain of dependent-latency loads otherwise).
__global__ __launch_bounds__(1024) void k_len_reduce(int nbins, int nslices, const unsigned* __restrict__ slices, u64* table)
{
    __shared__ u64 part[1024];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int v = blockIdx.x * 64 + lane;
    u64 a0 = 0, a1 = 0, a2 = 0, a3 = 0;
    if (v < nbins) {
        const unsigned* src = slices + v;
        int b = wave;
        for (; b + 48 < nslices; b += 64) {
            a0 += src[(size_t)b * nbins]; a1 += src[(size_t)(b + 16) * nbins];
            a2 += src[(size_t)(b + 32) * nbins]; a3 += src[(size_t)(b + 48) * nbins];
        }
        for (; b < nslices; b += 16) a0 += src[(size_t)b * nbins];
    }
    part[threadIdx.x] = (a0 + a1) + (a2 + a3);
    __syncthreads();
    if (wave == 0 && v < nbins) {
        u64 sum = 0;
        for (int w = 0; w < 16; ++w) sum += part[w * 64 + lane];
        table[v] = sum * (u64)v;
    }
}

// All bisection steps of search `c` from the table.
__device__ __forceinline__ void search_from_table(int c, int nbins, const u64* table, SearchState* st_, disco_policy* pol,
                                                  disco_search_out* sout)
{
    SearchState st = st_[c];
    disco_policy p = pol[c];
    while (st.step < st.n_steps) {
        const int L = p.l_th;
        const u64 s_pre = L <= 0 ? table[0] : (L < nbins ? table[L] : table[nbins]);
        const double A = st.which_acc == DISCO_ACC_SERVER_PREFILL_TOK ? (double)(i64)s_pre : (double)(i64)table[0];
        search_step(st, p, A, &sout[c]);
    }
    st_[c] = st;
    pol[c] = p;
}

// In place: table[L] = sum over v >= L of table[v], plus the lengths beyond
// the table; table[nbins] = those lengths alone.  One workgroup; with
// n_search > 0 its first threads then run the searches (thread = column).
__global__ __launch_bounds__(1024) void k_len_suffix(int nbins, u64* table, u64* other, int n_search, SearchState* st_,
                                                     disco_policy* pol, disco_search_out* sout)
{
    // Tiles of 8192 lengths from the top down: loaded coalesced into LDS, eight consecutive lengths per thread
    // (rows padded by one element per eight against bank conflicts), suffix scan of the thread totals, stored back
    // coalesced; `carry` = everything above the tile.
    constexpr int TILE = 8192;
    __shared__ u64 tile[TILE + TILE / 8];
    __shared__ u64 part[1024];
    __shared__ u64 carry_s;
    const int t = threadIdx.x;
    const u64 beyond = *other;
    u64 carry = beyond;
    for (int hi = nbins; hi > 0; hi -= TILE) {
        const int lo = hi > TILE ? hi - TILE : 0, len = hi - lo;
        for (int i = t; i < len; i += 1024) tile[i + (i >> 3)] = table[lo + i];
        __syncthreads();
        u64 sum = 0;
#pragma unroll
        for (int q = 0; q < 8; ++q) if (8 * t + q < len) sum += tile[9 * t + q];
        // suffix sums of the per-thread totals: within the wave by shuffles, across the 16 waves through LDS
        u64 incl = sum;
#pragma unroll
        for (int d = 1; d < 64; d <<= 1) {
            const unsigned lo32 = (unsigned)__shfl_down((int)(unsigned)incl, d, 64);
            const unsigned hi32 = (unsigned)__shfl_down((int)(unsigned)(incl >> 32), d, 64);
            if ((t & 63) + d < 64) incl += ((u64)hi32 << 32) | lo32;
        }
        if ((t & 63) == 0) part[t >> 6] = incl;     // the wave's total
        __syncthreads();
        u64 above = incl - sum + carry;             // the threads above this one in its wave
        for (int w = (t >> 6) + 1; w < 16; ++w) above += part[w];
#pragma unroll
        for (int q = 7; q >= 0; --q)
            if (8 * t + q < len) { above += tile[9 * t + q]; tile[9 * t + q] = above; }
        __syncthreads();
        for (int i = t; i < len; i += 1024) table[lo + i] = tile[i + (i >> 3)];
        if (t == 0) carry_s = tile[0];              // all lengths from `lo` up
        __syncthreads();
        carry = carry_s;
        __syncthreads();
    }
    if (threadIdx.x == 0) { table[nbins] = beyond; *other = 0; }
    if (n_search <= 0) return;
    __threadfence();                                // the table is read back by other threads of this workgroup
    __syncthreads();
    if ((int)threadIdx.x < n_search) search_from_table(threadIdx.x, nbins, table, st_, pol, sout);
}

unsigned dispatch_blocks(i64 units, i64 per_block)
{
    i64 b = (units + per_block - 1) / per_block;
    if (b > DP_MAX_BLOCKS) b = DP_MAX_BLOCKS;
    b /= disco_grid_divisor();
    if (b < 1) b = 1;
    return (unsigned)b;
}

bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

template <int G>
void launch_acc(const TraceView& v, const disco_policy* pol, int P, u64* part, const DispFin& fin,
                hipStream_t stream)
{
    const unsigned blocks = dispatch_blocks((v.n_req + 63) / 64, DP_WAVES);
    hipLaunchKernelGGL(k_dispatch_acc<G>, dim3(blocks), dim3(DP_BLOCK), 0, stream, v, pol, P, part, fin);
    hipLaunchKernelGGL(k_dispatch_fin, dim3(1), dim3(512), 0, stream, part, P, fin);
}

int pow2_cols(int P)
{
    int g = 1;
    while (g < P) g <<= 1;
    return g;
}

}  // namespace

void disco_launch_dispatch_acc(const TraceView& v, const disco_policy* pol, int P, u64* part, const DispFin& fin,
                               hipStream_t stream)
{
    switch (pow2_cols(P)) {
    case 1: {
        const unsigned blocks = dispatch_blocks((v.n_req + 3) / 4, DP_BLOCK);
        const bool vec = aligned16(v.l) && aligned16(v.n) && aligned16(v.s) && (!v.k || aligned16(v.k));
        if (vec) hipLaunchKernelGGL(k_dispatch_acc1<true>, dim3(blocks), dim3(DP_BLOCK), 0, stream, v, pol, part, fin);
        else hipLaunchKernelGGL(k_dispatch_acc1<false>, dim3(blocks), dim3(DP_BLOCK), 0, stream, v, pol, part, fin);
        hipLaunchKernelGGL(k_dispatch_fin, dim3(1), dim3(512), 0, stream, part, 1, fin);
        break;
    }
    case 2: launch_acc<2>(v, pol, P, part, fin, stream); break;
    case 4: launch_acc<4>(v, pol, P, part, fin, stream); break;
    case 8: launch_acc<8>(v, pol, P, part, fin, stream); break;
    case 16: launch_acc<16>(v, pol, P, part, fin, stream); break;
    case 32: launch_acc<32>(v, pol, P, part, fin, stream); break;
    default: launch_acc<64>(v, pol, P, part, fin, stream); break;
    }
}

void disco_launch_dispatch_mat(const TraceView& v, const disco_policy* pol, int P, uint8_t* decision, float* ttft,
                               hipStream_t stream)
{
    i64 b = (v.n_req + 255) / 256;
    if (b > 4096) b = 4096;
    if (b < 1) b = 1;
    hipLaunchKernelGGL(k_dispatch_mat, dim3((unsigned)b), dim3(256), 0, stream, v, pol, P, decision, ttft);
}

// table[L] = prompt tokens of the requests of length >= L for L < nbins, table[nbins] = those of longer requests
// (see k_len_hist).  `scratch` holds the workgroup slices; *other must be zero and is zero again afterwards.
static void launch_len_table(const TraceView& v, int nbins, unsigned* scratch, size_t scratch_bytes, u64* table, u64* other,
                             int n_search, SearchState* st, disco_policy* pol, disco_search_out* sout, hipStream_t stream)
{
    i64 blocks = (v.n_req + DP_BLOCK - 1) / DP_BLOCK;
    const i64 fit = (i64)(scratch_bytes / ((size_t)nbins * sizeof(unsigned)));
    if (blocks > fit) blocks = fit;
    if (blocks > DP_MAX_BLOCKS) blocks = DP_MAX_BLOCKS;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(k_len_hist, dim3((unsigned)blocks), dim3(DP_BLOCK), 0, stream, v, nbins, scratch, other);
    hipLaunchKernelGGL(k_len_reduce, dim3((unsigned)((nbins + 63) / 64)), dim3(1024), 0, stream, nbins, (int)blocks, scratch,
                       table);
    hipLaunchKernelGGL(k_len_suffix, dim3(1), dim3(1024), 0, stream, nbins, table, other, n_search, st, pol, sout);
}

void disco_launch_len_table(const TraceView& v, int nbins, unsigned* scratch, size_t scratch_bytes, u64* table, u64* other,
                            hipStream_t stream)
{
    launch_len_table(v, nbins, scratch, scratch_bytes, table, other, 0, nullptr, nullptr, nullptr, stream);
}

// Tabulated threshold search: the table, then every bisection step of every column from it (in the kernel that
// finishes the table).
void disco_launch_search_table(const TraceView& v, int n_search, int nbins, unsigned* scratch, size_t scratch_bytes,
                               u64* table, u64* other, SearchState* st, disco_policy* pol, disco_search_out* sout,
                               hipStream_t stream)
{
    launch_len_table(v, nbins, scratch, scratch_bytes, table, other, n_search, st, pol, sout, stream);
}

int disco_search_table_max_bins(void) { return LH_MAX_BINS; }
