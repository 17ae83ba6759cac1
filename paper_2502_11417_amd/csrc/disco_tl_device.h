// Device-side pieces shared by the token-timeline kernels (Sec. 4.3): wave
// scans of the running maximum, the column sets of a request, the class table
// of the TBT selection.
#pragma once
#include <math.h>

#include "disco_launch.h"
#include "disco_state.h"

namespace {

// ---------------------------------------------------------------- scans ----

// dpp_ctrl encodings (GFX9): row_shr:n = 0x110 + n, wave_shr:1 = 0x138.
template <int CTRL>
__device__ __forceinline__ float dpp_mov(float old, float src)
{
    return u2f((unsigned)__builtin_amdgcn_update_dpp((int)f2u(old), (int)f2u(src), CTRL, 0xF, 0xF, false));
}

// Inclusive running maximum over the 64 lanes: Hillis-Steele inside each row
// of 16 lanes with DPP row shifts (lanes whose source falls off the row keep
// -inf), then the three row totals are handed on through scalar registers.
__device__ __forceinline__ float wave_incl_max_dpp(float v, int lane)
{
    const float ninf = -INFINITY;
    v = fmaxf(v, dpp_mov<0x111>(ninf, v));
    v = fmaxf(v, dpp_mov<0x112>(ninf, v));
    v = fmaxf(v, dpp_mov<0x114>(ninf, v));
    v = fmaxf(v, dpp_mov<0x118>(ninf, v));
    const float t0 = bcast_f(v, 15), t1 = bcast_f(v, 31), t2 = bcast_f(v, 47);
    const float p1 = t0, p2 = fmaxf(t0, t1), p3 = fmaxf(p2, t2);
    const int row = lane >> 4;
    const float add = row == 0 ? ninf : (row == 1 ? p1 : (row == 2 ? p2 : p3));
    return fmaxf(v, add);
}

// Maximum over the wave, uniform.
__device__ __forceinline__ float wave_max_f32(float v)
{
    const float ninf = -INFINITY;
    v = fmaxf(v, dpp_mov<0x111>(ninf, v));
    v = fmaxf(v, dpp_mov<0x112>(ninf, v));
    v = fmaxf(v, dpp_mov<0x114>(ninf, v));
    v = fmaxf(v, dpp_mov<0x118>(ninf, v));
    return fmaxf(fmaxf(bcast_f(v, 15), bcast_f(v, 31)), fmaxf(bcast_f(v, 47), bcast_f(v, 63)));
}

// Value of the previous lane (lane 0 receives `first`).
__device__ __forceinline__ float wave_prev(float v, float first)
{
    return dpp_mov<0x138>(first, v);
}

// Loads the four arrival offsets of a lane: `g` is the global index of the
// lane's first element (a multiple of four elements away from a 16-byte
// boundary of the array); elements outside [0, n_tok) read as 0.
__device__ __forceinline__ void load4(const float* __restrict__ arr, i64 g, i64 n_tok, float r[4])
{
    if (g >= 0 && g + 3 < n_tok) {
        const float4 v = *reinterpret_cast<const float4*>(arr + g);
        r[0] = v.x; r[1] = v.y; r[2] = v.z; r[3] = v.w;
    } else {
#pragma unroll
        for (int k = 0; k < 4; ++k) r[k] = (g + k >= 0 && g + k < n_tok) ? arr[g + k] : 0.0f;
    }
}

// ---------------------------------------------------------- column sets ----

// Kinds of timeline of a (request, column) pair.
enum { TL_DEV = 0,        // device source
       TL_SRV = 1,        // server source, no hand-off
       TL_SRV_LAG = 2,    // server source with the lag trigger
       TL_SRV_BUF = 3,    // server source with the buffer hand-off (target: device)
       TL_DEV_BUF = 4,    // device source with the buffer hand-off (target: server)
       TL_KINDS = 5 };

// The column sets of a request by kind of timeline (lane = request).  The
// buffer hand-off (Sec. 4.3) applies when the source is the column's
// constrained endpoint.
__device__ __forceinline__ void request_sets(const disco_policy* sp, int P, int l, float s, float d, i64 i, u64 m[TL_KINDS])
{
    u64 m0 = 0ull, m1 = 0ull, m2 = 0ull, m3 = 0ull, m4 = 0ull;
    for (int j = 0; j < P; ++j) {
        unsigned dec; float t;
        dispatch_pair(sp[j], l, s, d, i, dec, t);
        const bool dev = (dec & 4u) != 0u;
        const int mg = sp[j].mig_mode, mode = sp[j].mode;
        const bool dev_constrained = mode == DISCO_MODE_DEVICE_CONSTRAINED || mode == DISCO_MODE_STOCH_DEVICE;
        const bool buf = mg == DISCO_MIG_BUFFER && (dev == dev_constrained);
        const u64 bit = 1ull << j;
        m4 |= (dev && buf) ? bit : 0ull;
        m0 |= (dev && !buf) ? bit : 0ull;
        m3 |= (!dev && buf) ? bit : 0ull;
        m2 |= (!dev && !buf && mg == DISCO_MIG_LAG) ? bit : 0ull;
        m1 |= (!dev && !buf && mg != DISCO_MIG_LAG) ? bit : 0ull;
    }
    m[TL_DEV] = m0; m[TL_SRV] = m1; m[TL_SRV_LAG] = m2; m[TL_SRV_BUF] = m3; m[TL_DEV_BUF] = m4;
}

// Pure pacing: a source whose constant gap is safely below tau (gap < 0.999 tau).
// Then u_0 = 0 and u_t = round(round(t gap) - t tau) < 0 for t >= 1 (the
// product's rounding error is below 2^-24 relative, far inside the 1e-3
// margin), the running maximum stays 0, delta_t = fma(t, tau, 0) = round(t tau),
// and no token is ever overdue.  The timeline depends on its length alone.
__device__ __forceinline__ bool pure_pacing(bool constant_gap, float gap, float tau)
{
    return constant_gap && gap < 0.999f * tau;
}

// Index of `mask` in a workgroup's copy of the class table (lane-private
// search over `ncls` entries), -1 if absent.
__device__ __forceinline__ int cls_find(const u64* s_cls, int ncls, u64 mask)
{
    int c = -1;
    for (int k = 0; k < ncls; ++k) c = (s_cls[k] == mask) ? k : c;
    return c;
}

// TBT selection key of a gap: its bit pattern minus key_lo (saturating at 0), clamped to key_cap.  Raw keys:
// key_lo = 0, key_cap = 0xFFFFFFFF.  Window mode: key_cap = 2^window; clamped keys (and the sign-flagged keys of
// tokens without a gap) have a bit above the window and match no prefix.
__device__ __forceinline__ unsigned tbt_key(unsigned bits, unsigned key_lo, unsigned key_cap)
{
    const unsigned off = __builtin_elementwise_sub_sat(bits, key_lo);
    return off < key_cap ? off : key_cap;
}

// Largest digit width whose `groups` histograms fit `words` bins.
__device__ __host__ __forceinline__ int fit_width(long groups, long words)
{
    int w = 0;
    while (w < 14 && (groups << (w + 1)) <= words) ++w;
    return w;
}

}  // namespace
