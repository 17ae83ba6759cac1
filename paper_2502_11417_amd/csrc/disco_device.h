// Device-side building blocks shared by the kernels of libdisco (gfx950, wave64).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include "disco.h"

typedef uint64_t u64;
typedef int64_t i64;

// Read-only view of a trace batch as the kernels see it.
struct TraceView {
    i64 n_req;
    const int32_t* l;      // prompt_len
    const int32_t* n;      // output_len
    const float* s;        // srv_ttft
    const float* tbt;      // srv_tbt (constant gap) or nullptr
    const float* k;        // dev_pre_spt or nullptr
    const float* g;        // dev_dec_spt or nullptr
    const i64* off;        // tok_off or nullptr
    const float* arr;      // tok_arr or nullptr
    float k_s, g_s, c;
};

__device__ __forceinline__ unsigned f2u(float x) { return __float_as_uint(x); }
__device__ __forceinline__ float u2f(unsigned x) { return __uint_as_float(x); }

// ---------------------------------------------------------------------------
// Counter-based random numbers: Philox4x32-10 (Salmon et al., SC'11), keyed by
// a 64-bit seed and counted by (element index, field).
// ---------------------------------------------------------------------------
struct Words { unsigned w0, w1, w2, w3; };

__device__ __forceinline__ Words philox4x32_10(u64 seed, u64 index, unsigned field)
{
    unsigned c0 = (unsigned)index, c1 = (unsigned)(index >> 32), c2 = field, c3 = 0u;
    unsigned k0 = (unsigned)seed, k1 = (unsigned)(seed >> 32);
#pragma unroll
    for (int r = 0; r < 10; ++r) {
        unsigned hi0 = __umulhi(0xD2511F53u, c0), lo0 = 0xD2511F53u * c0;
        unsigned hi1 = __umulhi(0xCD9E8D57u, c2), lo1 = 0xCD9E8D57u * c2;
        unsigned n0 = hi1 ^ c1 ^ k0, n2 = hi0 ^ c3 ^ k1;
        c0 = n0; c1 = lo1; c2 = n2; c3 = lo0;
        k0 += 0x9E3779B9u; k1 += 0xBB67AE85u;
    }
    return Words{c0, c1, c2, c3};
}

// 23 random bits to a uniform on (0,1): (x >> 9 + 1/2) 2^-23, exact in fp32.
__device__ __forceinline__ float u23(unsigned x)
{
    return __fmaf_rn((float)(x >> 9), 0x1p-23f, 0x1p-24f);
}

// Uniform variate of request i in run `run` of the stochastic baselines
// (Sec. 5.1): key = (run, tag), counter = (i, field 6), word 0.
__device__ __forceinline__ float route_uniform(int run, i64 i)
{
    const u64 seed = ((u64)0x53544F43u << 32) | (u64)(unsigned)run;
    return u23(philox4x32_10(seed, (u64)i, 6u).w0);
}

// ---------------------------------------------------------------------------
// Dispatch of one (request, column) pair: Sec. 4.2, Alg. 2 (wait time) and
// Alg. 3 (length threshold).  Both modes are evaluated branch-free so that
// lanes holding different columns stay converged.  The stochastic baselines
// of Sec. 5.1 (modes 2 and 3: one endpoint per request, the constrained one
// with probability beta) take a branch of their own: their draw costs ten
// times a pair of the method.  i = index of the request in the trace.
//   decision bit0 = server started, bit1 = device started, bit2 = device won.
// ---------------------------------------------------------------------------
//   u (dispatch_pair_u): the uniform variate of (run, request) when the caller has drawn it already.
__device__ __forceinline__ void dispatch_pair_u(const disco_policy& p, int l, float s, float d, i64 i, bool have_u, float u,
                                                unsigned& decision, float& ttft)
{
    if (p.mode >= DISCO_MODE_STOCH_SERVER) {
        const bool constrained = (have_u ? u : route_uniform(p.l_mid, i)) < p.beta;
        const bool to_server = (p.mode == DISCO_MODE_STOCH_SERVER) ? constrained : !constrained;
        decision = to_server ? 1u : 6u;
        ttft = to_server ? s : d;
        return;
    }
    // device-constrained wait (Eq. 1 united with Alg. 2's step map)
    float ramp = p.beta * (float)l;
    float w = (ramp < p.w_tail) ? ramp : p.w_tail;     // a NaN ramp falls through to w_tail
    w = (l == p.l_mid) ? p.w_mid : w;
    w = (l <= p.l_th) ? 0.0f : w;
    bool d_started = s > w;                             // strict: a server token at exactly w cancels the device
    float x = w + d;
    bool d_win = d_started && (x < s);                  // ties go to the server
    unsigned d_dec = 1u | (d_started ? 2u : 0u) | (d_win ? 4u : 0u);
    float d_ttft = d_win ? x : s;
    // server-constrained threshold (Alg. 3: strict l < l_th runs on the device alone)
    bool dev_only = l < p.l_th;
    bool s_win = dev_only || (d < s);
    unsigned s_dec = dev_only ? 6u : (s_win ? 7u : 3u);
    float s_ttft = s_win ? d : s;
    bool srv_mode = (p.mode == DISCO_MODE_SERVER_CONSTRAINED);
    decision = srv_mode ? s_dec : d_dec;
    ttft = srv_mode ? s_ttft : d_ttft;
}

__device__ __forceinline__ void dispatch_pair(const disco_policy& p, int l, float s, float d, i64 i,
                                              unsigned& decision, float& ttft)
{
    dispatch_pair_u(p, l, s, d, i, false, 0.0f, decision, ttft);
}

// ---------------------------------------------------------------------------
// Wave-level helpers (64 lanes).
// ---------------------------------------------------------------------------
__device__ __forceinline__ float wave_incl_max(float v, int lane)
{
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
        float o = __shfl_up(v, d, 64);
        if (lane >= d) v = fmaxf(v, o);
    }
    return v;
}

__device__ __forceinline__ float bcast_f(float v, int src_lane)
{
    return u2f((unsigned)__builtin_amdgcn_readlane((int)f2u(v), src_lane));
}
__device__ __forceinline__ int bcast_i(int v, int src_lane)
{
    return __builtin_amdgcn_readlane(v, src_lane);
}

__device__ __forceinline__ u64 shfl_xor_u64(u64 v, int m)
{
    unsigned lo = (unsigned)v, hi = (unsigned)(v >> 32);
    lo = (unsigned)__shfl_xor((int)lo, m, 64);
    hi = (unsigned)__shfl_xor((int)hi, m, 64);
    return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ u64 shfl_down_u64(u64 v, int d)
{
    unsigned lo = (unsigned)v, hi = (unsigned)(v >> 32);
    lo = (unsigned)__shfl_down((int)lo, d, 64);
    hi = (unsigned)__shfl_down((int)hi, d, 64);
    return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ double shfl_xor_f64(double v, int m)
{
    return __longlong_as_double((long long)shfl_xor_u64((u64)__double_as_longlong(v), m));
}

// Wave-wide reductions with DPP row shifts (row = 16 lanes): four shifted
// adds leave each row's total in its last lane; the four row totals are then
// combined through scalar registers.  The order of the additions is fixed, so
// floating-point sums are reproducible.  The result is uniform over the wave.
template <int CTRL>
__device__ __forceinline__ unsigned dpp_u32(unsigned old, unsigned src)
{
    return (unsigned)__builtin_amdgcn_update_dpp((int)old, (int)src, CTRL, 0xF, 0xF, false);
}
template <int CTRL>
__device__ __forceinline__ u64 dpp_u64(u64 src)      // lanes without a source receive 0
{
    const unsigned lo = dpp_u32<CTRL>(0u, (unsigned)src);
    const unsigned hi = dpp_u32<CTRL>(0u, (unsigned)(src >> 32));
    return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ u64 bcast_u64(u64 v, int lane)
{
    const unsigned lo = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)v, lane);
    const unsigned hi = (unsigned)__builtin_amdgcn_readlane((int)(unsigned)(v >> 32), lane);
    return ((u64)hi << 32) | lo;
}
__device__ __forceinline__ u64 wave_sum_u64(u64 v)
{
    v += dpp_u64<0x111>(v); v += dpp_u64<0x112>(v); v += dpp_u64<0x114>(v); v += dpp_u64<0x118>(v);
    return bcast_u64(v, 15) + bcast_u64(v, 31) + bcast_u64(v, 47) + bcast_u64(v, 63);
}
__device__ __forceinline__ double wave_sum_f64(double x)
{
    u64 b = (u64)__double_as_longlong(x);
    // +0.0 has the all-zero pattern, so the zero fill of dpp_u64 is the additive identity
    x += __longlong_as_double((long long)dpp_u64<0x111>(b)); b = (u64)__double_as_longlong(x);
    x += __longlong_as_double((long long)dpp_u64<0x112>(b)); b = (u64)__double_as_longlong(x);
    x += __longlong_as_double((long long)dpp_u64<0x114>(b)); b = (u64)__double_as_longlong(x);
    x += __longlong_as_double((long long)dpp_u64<0x118>(b)); b = (u64)__double_as_longlong(x);
    const double r0 = __longlong_as_double((long long)bcast_u64(b, 15)), r1 = __longlong_as_double((long long)bcast_u64(b, 31));
    const double r2 = __longlong_as_double((long long)bcast_u64(b, 47)), r3 = __longlong_as_double((long long)bcast_u64(b, 63));
    return ((r0 + r1) + r2) + r3;
}
__device__ __forceinline__ unsigned wave_min_u32(unsigned v)
{
    v = min(v, dpp_u32<0x111>(0xFFFFFFFFu, v)); v = min(v, dpp_u32<0x112>(0xFFFFFFFFu, v));
    v = min(v, dpp_u32<0x114>(0xFFFFFFFFu, v)); v = min(v, dpp_u32<0x118>(0xFFFFFFFFu, v));
    return min(min((unsigned)bcast_i((int)v, 15), (unsigned)bcast_i((int)v, 31)),
               min((unsigned)bcast_i((int)v, 47), (unsigned)bcast_i((int)v, 63)));
}
__device__ __forceinline__ unsigned wave_max_u32(unsigned v)
{
    v = max(v, dpp_u32<0x111>(0u, v)); v = max(v, dpp_u32<0x112>(0u, v));
    v = max(v, dpp_u32<0x114>(0u, v)); v = max(v, dpp_u32<0x118>(0u, v));
    return max(max((unsigned)bcast_i((int)v, 15), (unsigned)bcast_i((int)v, 31)),
               max((unsigned)bcast_i((int)v, 47), (unsigned)bcast_i((int)v, 63)));
}

// ---------------------------------------------------------------------------
// Unified cost (Sec. 4.1, App. E): written one fp64 operation at a time, in
// the order server = a + b, energy = c + d, total = server + lambda * energy.
// ---------------------------------------------------------------------------
__device__ __forceinline__ double server_cost_of(const disco_cost_params& c, i64 s_pre, i64 s_dec)
{
    double a = c.cs_pre * (double)s_pre;
    double b = c.cs_dec * (double)s_dec;
    return a + b;
}
__device__ __forceinline__ double device_energy_of(const disco_cost_params& c, i64 d_pre, i64 d_dec)
{
    double a = c.e_pre * (double)d_pre;
    double b = c.e_dec * (double)d_dec;
    return a + b;
}
