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
__device__ __forceinline__ PairResult pair_eval(const disco_policy& p, int l, float s, float d, i64 i)
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
        dispatch_pair(p, l, s, d, i, dec, t);
        r.srv_started = (dec & 1u) != 0u;
        r.dev_started = (dec & 2u) != 0u;
        r.dev_win = (dec & 4u) != 0u;
        r.ttft = t;
    }
    return r;
}

__device__ __forceinline__ int table_mode(const disco_policy& p, bool colv)
{
    const bool any_d = __ballot(colv && p.mode == DISCO_MODE_DEVICE_CONSTRAINED) != 0ull;
    const bool any_s = __ballot(colv && p.mode == DISCO_MODE_SERVER_CONSTRAINED) != 0ull;
    const bool any_x = __ballot(colv && p.mode >= DISCO_MODE_STOCH_SERVER) != 0ull;
    return any_x ? 2 : (any_d ? (any_s ? 2 : 1) : 0);
}

}  // namespace
