// Per-pair dispatch evaluation specialised on the kind of policy table, and
// the LDS staging record of the dispatch-type passes.
#pragma once
#include "disco_device.h"

namespace {

constexpr int DP_BLOCK = 1024;
constexpr int DP_WAVES = DP_BLOCK / 64;
constexpr int DP_MAX_BLOCKS = 256;          // one workgroup per CU: the ticket chain stays short

struct Staged { int l; float s; int n; float d; };      // 16 bytes, one per request of the batch
// What a race decides does not depend on the column: d = device TTFT, m = TTFT of a race (ties go to the server), pn = decode
// tokens with a count of one above them (n < 2^16, so 64 of them add up below bit 22), and, in an array of its
// own, pnr = pn if the device wins the race, else 0.  A threshold column (Alg. 3) only selects between the
// device-only and the race values.
struct StagedRace { int l; unsigned d, m, pn; };         // d, m: bit patterns of the two TTFT candidates
constexpr unsigned PN_COUNT_SHIFT = 22;

// ------------------------------------------------------------ per pair ----

struct PairResult { bool srv_started, dev_started, dev_win; float ttft; };

// MODE 0: every column is server-constrained (Alg. 3), 1: every column is
// device-constrained (Alg. 2 / Eq. 1), 2: mixed table or stochastic baseline columns.
template <int MODE>
__device__ __forceinline__ PairResult pair_eval(const disco_policy& p, int l, float s, float d, i64 i, bool have_u = false,
                                                float u = 0.0f)
{
    PairResult r;
    if (MODE == 0) {
        const bool dev_only = l < p.l_th;               // strict: Alg. 3
        r.srv_started = !dev_only;
        r.dev_started = true;
        r.dev_win = dev_only || (d < s);                // ties go to the server
        r.ttft = r.dev_win ? d : s;
    } else if (MODE == 1) {
        float ramp = p.beta * (float)l;
        float w = (ramp < p.w_tail) ? ramp : p.w_tail;  // a NaN ramp falls through to w_tail
        w = (l == p.l_mid) ? p.w_mid : w;
        w = (l <= p.l_th) ? 0.0f : w;
        const float x = w + d;
        r.srv_started = true;
        r.dev_started = s > w;                          // a server token at exactly w cancels the device
        r.dev_win = r.dev_started && (x < s);
        r.ttft = r.dev_win ? x : s;
    } else {
        unsigned dec; float t;
        dispatch_pair_u(p, l, s, d, i, have_u, u, dec, t);
        r.srv_started = (dec & 1u) != 0u;
        r.dev_started = (dec & 2u) != 0u;
        r.dev_win = (dec & 4u) != 0u;
        r.ttft = t;
    }
    return r;
}

// Stochastic baseline columns (Sec. 5.1) of the same run share the uniform variate of a request: the levels of a
// run are nested.  Per wave (lane = column): up to STOCH_SHARE distinct runs among the columns, lane k keeps run
// k.  Per batch of 64 requests every lane draws the variates of the request it loaded (lane = request), one per
// run; a column lane then fetches the variate of (its run, the request it evaluates) from the lane that holds it:
// R draws per request instead of one per (request, column) pair.
constexpr int STOCH_SHARE = 8;
struct StochRuns { int R; int ridx; int run_of_lane; bool on; };     // on: some stochastic column, at most STOCH_SHARE runs

__device__ __forceinline__ StochRuns stoch_runs(const disco_policy& p, bool colv, int lane)
{
    const bool st = colv && p.mode >= DISCO_MODE_STOCH_SERVER;
    u64 todo = __ballot(st);
    StochRuns s{0, -1, 0, todo != 0ull};
    while (todo) {
        const int leader = __ffsll((long long)todo) - 1;
        const int r0 = bcast_i(p.l_mid, leader);
        const u64 same = __ballot(st && p.l_mid == r0);
        if (st && p.l_mid == r0) s.ridx = s.R;
        if (lane == s.R) s.run_of_lane = r0;
        s.R += 1;
        todo &= ~same;
    }
    if (s.R > STOCH_SHARE) s.on = false;
    return s;
}

// lane = request i of the batch
__device__ __forceinline__ void stoch_draw(const StochRuns& s, i64 i, float u[STOCH_SHARE])
{
#pragma unroll
    for (int k = 0; k < STOCH_SHARE; ++k)
        if (k < s.R) u[k] = route_uniform(bcast_i(s.run_of_lane, k), i);
}

// the variate of (this lane's run, the request that lane `src` holds); UNIFORM: `src` is the same in every lane
template <bool UNIFORM>
__device__ __forceinline__ float stoch_fetch(const StochRuns& s, const float u[STOCH_SHARE], int src)
{
    float x = 0.0f;
#pragma unroll
    for (int k = 0; k < STOCH_SHARE; ++k)
    {
        const float v = UNIFORM ? bcast_f(u[k], src) : __shfl(u[k], src, 64);
        x = (k == s.ridx) ? v : x;
    }
    return x;
}

__device__ __forceinline__ int table_mode(const disco_policy& p, bool colv)
{
    const bool any_d = __ballot(colv && p.mode == DISCO_MODE_DEVICE_CONSTRAINED) != 0ull;
    const bool any_s = __ballot(colv && p.mode == DISCO_MODE_SERVER_CONSTRAINED) != 0ull;
    const bool any_x = __ballot(colv && p.mode >= DISCO_MODE_STOCH_SERVER) != 0ull;
    return any_x ? 2 : (any_d ? (any_s ? 2 : 1) : 0);
}

}  // namespace
