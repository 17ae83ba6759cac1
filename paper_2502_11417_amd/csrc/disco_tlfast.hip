// Token timelines (Sec. 4.3): the class-mode TBT histogram passes of
// disco_reduce_stats and what prepares them once per selection.
//
//   k_tl_assign  lane = request: timelines that the token walk's summaries
//                prove analytic (running maximum never left 0, so
//                delta_t = round(t tau)) are counted per class and length;
//                the others get their histogram row into the request's
//                descriptor and the request into the walk list
//   k_pp_reduce  per-workgroup count slices -> counts per class and length
//   k_tl_hist    one pass over the walk list (workgroup body and walker in
//                disco_tl_hist_fast.h): a wave walks one request at a time in
//                chunks of 256 tokens, four consecutive tokens per lane (one
//                16-byte load per lane and chunk, the next chunk's load
//                issued before the current one is used)
//
// The delivery recurrence delta_t = max(r_t, delta_{t-1} + tau) is evaluated
// in the shifted domain u_t = r_t - t tau, where it is a running maximum M_t
// and delta_t = fma(t, tau, M_t).  `max` is exact and associative, so any
// evaluation order gives the sequential definition bit for bit.  The
// histogram walk needs M_t per token: a 4-element scan in registers and a DPP
// scan across the wave; the gaps delta_t - delta_{t-1} go to the LDS
// histogram of the timeline's class.
//
// Lag trigger (token t is overdue by more than kappa tau): evaluated exactly,
// one IEEE fp32 operation at a time in the order of the definition (slot =
// delta_{t-1} + tau, lag = r_t - slot), in every chunk that passes a cheap necessary
// condition (see walk_hist); the other chunks provably cannot trigger.
//
// A timeline is computed once per request and source, never per policy
// column: the recurrence does not depend on the pair's TTFT, so every column
// only picks the timeline of its dispatch winner.
#include <string.h>

#include "disco_tl_hist_fast.h"

namespace {


// Analytic timelines per class and length, counted per workgroup in LDS (two 16-bit counts per word, a workgroup
// sees at most 65535 requests) for the first PP_LDS_CLS classes and stored as one slice per workgroup; classes
// beyond that (tables of many columns) are counted in device memory directly.
constexpr int PP_LDS_CLS = 16;
constexpr int PP_WORDS = DISCO_PP_NMAX / 2 + 1;              // words per class: lengths 0 .. DISCO_PP_NMAX
constexpr int AS_BLOCK = 1024;

__global__ __launch_bounds__(AS_BLOCK) void k_tl_assign(TraceView tr, const disco_policy* __restrict__ pol, int P,
                                                        const TlSummary* __restrict__ summary,
                                                        const BufSummary* __restrict__ bufsum, SelState* S,
                                                        u64* __restrict__ desc_out, unsigned* __restrict__ list,
                                                        unsigned* __restrict__ slices, unsigned* __restrict__ ppcnt,
                                                        unsigned* __restrict__ dhist, int use_lds)
{
    __shared__ unsigned cnt[PP_LDS_CLS * PP_WORDS];          // 128 KB
    __shared__ unsigned s_nw[2], s_base[2];                  // [0] long requests (front of the list), [1] the others (back)
    __shared__ u64 s_cls[DISCO_MAX_CLS];
    __shared__ signed char s_slot[DISCO_MAX_CLS];
    __shared__ disco_policy spol[DISCO_MAX_COLS];
    const TlSel* tl = &S->tl;
    if (tl->fallback) return;                                // per-slot histograms: the general kernel walks everything
    const int ncls = tl->ncls;
    const int nlds = use_lds ? (ncls < PP_LDS_CLS ? ncls : PP_LDS_CLS) : 0;
    if ((int)threadIdx.x < P) spol[threadIdx.x] = pol[threadIdx.x];
    if (threadIdx.x < DISCO_MAX_CLS) { s_cls[threadIdx.x] = tl->cls_mask[threadIdx.x]; s_slot[threadIdx.x] = tl->cls_slot[threadIdx.x]; }
    for (int i = threadIdx.x; i < nlds * PP_WORDS; i += AS_BLOCK) cnt[i] = 0u;
    if (threadIdx.x < 2) s_nw[threadIdx.x] = 0u;
    __syncthreads();
    const int lane = threadIdx.x & 63;
    // a contiguous share of the requests per workgroup (at most 65535, see the launch)
    const i64 per = (tr.n_req + gridDim.x - 1) / gridDim.x;
    const i64 lo = (i64)blockIdx.x * per;
    const i64 hi = lo + per < tr.n_req ? lo + per : tr.n_req;
    u64 wmask = 0ull, lmask = 0ull;                          // bit r: this thread's request of round r has tokens to walk / is long
    int round = 0;
    for (i64 i = lo + threadIdx.x; i < hi; i += AS_BLOCK, ++round) {
        const int l = tr.l[i], n = tr.n[i];
        const float s = tr.s[i];
        const float k = tr.k ? tr.k[i] : tr.k_s;
        const TlSummary sm = summary[i];
        u64 m[TL_KINDS];
        request_sets(spol, P, l, s, __fmaf_rn((float)l, k, tr.c), i, m);
        u64 desc = DESC_NONE5;
        BufSummary bs{0.0f, -1, 0, 0, 0.0f, -1, 0, 0};
        if ((m[TL_SRV_BUF] | m[TL_DEV_BUF]) != 0ull) {
            bs = bufsum[i];
            // migrated requests by number of delayed tokens, per column (those without one are implied by the
            // migration count)
#pragma unroll
            for (int kind = TL_SRV_BUF; kind <= TL_DEV_BUF; ++kind) {
                const int me = kind == TL_SRV_BUF ? bs.m_s : bs.m_d;
                const int dl = kind == TL_SRV_BUF ? bs.delay_s : bs.delay_d;
                if (m[kind] == 0ull || summary_m(me) < 0 || dl <= 0) continue;
                const int bin = dl < DISCO_DELAY_BINS - 1 ? dl : DISCO_DELAY_BINS - 1;
                for (u64 left = m[kind]; left != 0ull; left &= left - 1ull)
                    atomicAdd(&dhist[(size_t)(__ffsll((long long)left) - 1) * DISCO_DELAY_BINS + bin], 1u);
            }
        }
#pragma unroll
        for (int kind = 0; kind < TL_KINDS; ++kind) {
            if (m[kind] == 0ull) continue;
            const int c = cls_find(s_cls, ncls, m[kind]);
            if (c < 0) { S->tl.error = 1; continue; }        // a set the classification did not see: never expected
            if (kind < TL_SRV_BUF ? timeline_is_analytic(kind, n, sm) : buf_timeline_is_analytic(kind, n, bs)) {
                if (c < nlds) atomicAdd(&cnt[c * PP_WORDS + (n >> 1)], 1u << (16 * (n & 1)));
                else atomicAdd(&ppcnt[(size_t)c * (DISCO_PP_NMAX + 1) + n], 1u);
            } else {
                const int sl = s_slot[c];
                if (sl < 0) { S->tl.error = 1; continue; }
                desc = (desc & ~(0xFFull << (8 * kind))) | ((u64)(unsigned)sl << (8 * kind));
            }
        }
        desc_out[i] = desc;
        const bool walk = desc != DESC_NONE5, lng = n >= WALK_LONG_TOKENS;
        if (walk) wmask |= 1ull << round;
        if (walk && lng) lmask |= 1ull << round;
        const u64 wb = __ballot(walk);
        if (wb) {
            const u64 lb = __ballot(walk && lng);
            if (lane == __ffsll((long long)wb) - 1) {
                if (lb) atomicAdd(&s_nw[0], (unsigned)__popcll(lb));
                if (wb & ~lb) atomicAdd(&s_nw[1], (unsigned)__popcll(wb & ~lb));
            }
        }
    }
    __syncthreads();
    // the requests with tokens to walk go to a device-wide list (any order: the histograms are sums), a range of it
    // per workgroup
    const unsigned nw0 = s_nw[0], nw1 = s_nw[1];
    __syncthreads();
    if (threadIdx.x == 0) {
        s_base[0] = nw0 ? atomicAdd(&S->tl.nlist, nw0) : 0u;
        s_base[1] = nw1 ? atomicAdd(&S->tl.nlist_back, nw1) : 0u;
        s_nw[0] = 0u; s_nw[1] = 0u;
    }
    __syncthreads();
    if (nw0 | nw1) {
        round = 0;
        for (i64 i = lo + threadIdx.x; i < hi; i += AS_BLOCK, ++round) {
            const bool w = (wmask >> round) & 1ull, lng = (lmask >> round) & 1ull;
            const u64 wb = __ballot(w);
            if (!wb) continue;
            const u64 lb = __ballot(w && lng), sb = wb & ~lb;
            const int leader = __ffsll((long long)wb) - 1;
            unsigned at0 = 0u, at1 = 0u;
            if (lane == leader) {
                if (lb) at0 = atomicAdd(&s_nw[0], (unsigned)__popcll(lb));
                if (sb) at1 = atomicAdd(&s_nw[1], (unsigned)__popcll(sb));
            }
            at0 = (unsigned)bcast_i((int)at0, leader);
            at1 = (unsigned)bcast_i((int)at1, leader);
            const u64 below = (1ull << lane) - 1ull;
            if (w && lng) list[s_base[0] + at0 + (unsigned)__popcll(lb & below)] = (unsigned)i;
            if (w && !lng) list[(size_t)tr.n_req - 1 - (s_base[1] + at1 + (unsigned)__popcll(sb & below))] = (unsigned)i;
        }
    }
    unsigned* mine = slices + (size_t)blockIdx.x * PP_LDS_CLS * PP_WORDS;
    for (int i = threadIdx.x; i < nlds * PP_WORDS; i += AS_BLOCK) mine[i] = cnt[i];
}

// ppcnt[c][n] += sum over the workgroup slices.  Workgroup = (class, 256 words of two lengths each); four groups
// of threads share the slices and meet in LDS.
__global__ __launch_bounds__(1024) void k_pp_reduce(const SelState* S, int nslices, const unsigned* __restrict__ slices,
                                                    unsigned* __restrict__ ppcnt, int use_lds)
{
    __shared__ unsigned part[2][1024];
    const TlSel* tl = &S->tl;
    const int c = blockIdx.x;
    if (tl->fallback || !use_lds || c >= tl->ncls || c >= PP_LDS_CLS) return;
    const int w = blockIdx.y * 256 + (threadIdx.x & 255), grp = threadIdx.x >> 8;
    unsigned even = 0u, odd = 0u;
    if (w < PP_WORDS) {
#pragma unroll 8
        for (int b = grp; b < nslices; b += 4) {
            const unsigned v = slices[((size_t)b * PP_LDS_CLS + c) * PP_WORDS + w];
            even += v & 0xFFFFu; odd += v >> 16;
        }
    }
    part[0][threadIdx.x] = even; part[1][threadIdx.x] = odd;
    __syncthreads();
    if (grp == 0 && w < PP_WORDS) {
        for (int g = 1; g < 4; ++g) { even += part[0][threadIdx.x + 256 * g]; odd += part[1][threadIdx.x + 256 * g]; }
        unsigned* row = ppcnt + (size_t)c * (DISCO_PP_NMAX + 1);
        if (even) row[2 * w] += even;
        if (odd && 2 * w + 1 <= DISCO_PP_NMAX) row[2 * w + 1] += odd;
    }
}

// One histogram pass over the walk list (regular passes; the spare passes run the same body in the kernel that
// also advances the selection).
__global__ __launch_bounds__(TH_BLOCK, 8) void k_tl_hist(TraceView tr, i64 n_tok, int align, HistArgs a)
{
    __shared__ __align__(16) unsigned smem[DISCO_TL_HIST_WORDS];
    tl_hist_fast_body(smem, tr, n_tok, align, a, blockIdx.x, gridDim.x);
}

}  // namespace

// Once per selection, after the classification: descriptors of all requests, analytic timelines counted per class
// and length.  `slices`: scratch for the workgroup slices (slices_bytes).
void disco_launch_tl_assign(const TraceView& v, const disco_policy* pol, int P, const void* summary, SelState* S,
                            const void* bufsum, u64* desc, unsigned* list, unsigned* slices, size_t slices_bytes,
                            unsigned* ppcnt, unsigned* dhist, hipStream_t stream)
{
    if (v.n_req <= 0) return;
    i64 b = (v.n_req + 49151) / 49152;             // at most 65535 requests per workgroup: 16-bit counts in LDS
    if (b < 250) b = 250;                          // one workgroup per CU (128 KB of LDS each); at most 64 rounds per thread
    const i64 fit = (i64)(slices_bytes / ((size_t)PP_LDS_CLS * PP_WORDS * sizeof(unsigned)));
    int use_lds = 1;
    // tens of millions of requests (or the testing aid that shrinks the grids): counts in device memory
    if (b > fit || disco_grid_divisor() > 1) { b = (v.n_req + 65535) / 65536; use_lds = 0; }
    hipLaunchKernelGGL(k_tl_assign, dim3((unsigned)b), dim3(AS_BLOCK), 0, stream, v, pol, P, (const TlSummary*)summary,
                       (const BufSummary*)bufsum, S, desc, list, slices, ppcnt, dhist, use_lds);
    hipLaunchKernelGGL(k_pp_reduce, dim3(PP_LDS_CLS, (PP_WORDS + 255) / 256), dim3(1024), 0, stream, (const SelState*)S, (int)b, (const unsigned*)slices,
                       ppcnt, use_lds);
}

void disco_launch_tl_hist_fast(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a,
                               hipStream_t stream)
{
    (void)pol;
    HistArgs h;
    memset(&h, 0, sizeof(h));
    h.tau = a.tau; h.kt = a.kt; h.P = a.P; h.pass = a.pass;
    h.S = a.S; h.ghist = a.ghist;
    h.desc = a.desc; h.list = a.list;
    i64 b = (v.n_req + TH_BLOCK / 64 - 1) / (TH_BLOCK / 64);      // at most one request per wave
    if (b < 1) b = 1;
    if (b > 512) b = 512;                                          // two resident workgroups per CU
    b /= disco_grid_divisor();
    if (b < 1) b = 1;
    const int align = (int)(((uintptr_t)v.arr >> 2) & 3);
    hipLaunchKernelGGL(k_tl_hist, dim3((unsigned)b), dim3(TH_BLOCK), 0, stream, v, n_tok, align, h);
}
