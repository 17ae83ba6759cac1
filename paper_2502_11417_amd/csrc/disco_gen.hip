// disco_gen_trace: synthetic trace on the device.
//
// Stand-in for the measured server traces and device profiles of Sec. 5.1;
// the recipe (log-normal prompt length and server TTFT, server TTFT
// independent of prompt length, device TTFT linear in it) follows Sec. 3 and
// the scalability study of Sec. 5.3.  Random numbers come from Philox4x32-10
// (Salmon et al., SC'11) keyed by the seed and counted by (element index,
// field), so every element is independent of the launch geometry.  The
// elementary functions are fixed sequences of IEEE fp32 operations, which
// makes the trace reproducible bit for bit by any other implementation of the
// same definition.
#include "disco_common.h"
#include "disco_device.h"

namespace {

// ln of a positive normal number: x = 2^e m with m in (sqrt(1/2), sqrt(2)],
// ln m = 2 atanh(s), s = (m - 1) / (m + 1), odd series through s^11.
__device__ __forceinline__ float gen_ln(float x)
{
    unsigned bits = f2u(x);
    int e = (int)(bits >> 23) - 127;
    float m = u2f((bits & 0x007FFFFFu) | 0x3F800000u);
    if (m > 1.41421354f) { m = m * 0.5f; e = e + 1; }
    float f = m - 1.0f;
    float s = __fdiv_rn(f, 2.0f + f);
    float z = s * s;
    float p = __fmaf_rn(z, 0.181818187f, 0.222222224f);
    p = __fmaf_rn(z, p, 0.285714298f);
    p = __fmaf_rn(z, p, 0.400000006f);
    p = __fmaf_rn(z, p, 0.666666687f);
    float sz = s * z;
    float lnm = __fmaf_rn(sz, p, 2.0f * s);
    return __fmaf_rn((float)e, 0.693147182f, lnm);
}

// exp on [-86, 88]: n = rint(x log2 e), r = x - n ln 2 (two-part ln 2),
// series of e^r through r^7, exact scaling by 2^n.
__device__ __forceinline__ float gen_exp(float x)
{
    x = (x < -86.0f) ? -86.0f : x;
    x = (x > 88.0f) ? 88.0f : x;
    float t = x * 1.44269502f;
    float n = rintf(t);
    float r = __fmaf_rn(n, -0.693145752f, x);
    r = __fmaf_rn(n, -1.42860677e-06f, r);
    float p = __fmaf_rn(r, 1.98412701e-04f, 1.38888892e-03f);
    p = __fmaf_rn(r, p, 8.33333377e-03f);
    p = __fmaf_rn(r, p, 4.16666679e-02f);
    p = __fmaf_rn(r, p, 0.166666672f);
    p = __fmaf_rn(r, p, 0.5f);
    p = __fmaf_rn(r, p, 1.0f);
    p = __fmaf_rn(r, p, 1.0f);
    int ni = (int)n;
    float scale = u2f((unsigned)(ni + 127) << 23);
    return p * scale;
}

// cos(2 pi u), u in (0,1): quadrant q = rint(4u), v = u - q/4 exactly,
// a = 2 pi v in [-pi/4, pi/4], series of cos and sin.
__device__ __forceinline__ float gen_cos2pi(float u)
{
    float q = rintf(4.0f * u);
    float v = __fmaf_rn(q, -0.25f, u);
    float a = v * 6.28318548f;
    float a2 = a * a;
    float c = __fmaf_rn(a2, -2.75573200e-07f, 2.48015876e-05f);
    c = __fmaf_rn(a2, c, -1.38888892e-03f);
    c = __fmaf_rn(a2, c, 4.16666679e-02f);
    c = __fmaf_rn(a2, c, -0.5f);
    c = __fmaf_rn(a2, c, 1.0f);
    float s = __fmaf_rn(a2, -2.50521079e-08f, 2.75573188e-06f);
    s = __fmaf_rn(a2, s, -1.98412701e-04f);
    s = __fmaf_rn(a2, s, 8.33333377e-03f);
    s = __fmaf_rn(a2, s, -0.166666672f);
    s = __fmaf_rn(a2, s, 1.0f);
    s = s * a;
    int qi = (int)q & 3;
    float res = (qi & 1) ? s : c;
    // q = 0: c, 1: -s, 2: -c, 3: s
    return (qi == 1 || qi == 2) ? -res : res;
}

__device__ __forceinline__ float gen_normal(unsigned w0, unsigned w1)
{
    float rad = sqrtf(-2.0f * gen_ln(u23(w0)));   // IEEE-rounded square root
    return rad * gen_cos2pi(u23(w1));
}

__device__ __forceinline__ float gen_lognormal(unsigned w0, unsigned w1, float mu, float sigma)
{
    return gen_exp(__fmaf_rn(sigma, gen_normal(w0, w1), mu));
}

__device__ __forceinline__ int floor_clamp(float v, int lo, int hi)
{
    float f = floorf(v);
    f = (f < (float)lo) ? (float)lo : f;
    f = (f > (float)hi) ? (float)hi : f;
    return (int)f;
}

enum { F_PROMPT = 0, F_OUTPUT = 1, F_TTFT = 2, F_TBT = 3, F_DEVICE = 4, F_GAP = 5 };

__global__ __launch_bounds__(256) void k_gen_requests(disco_gen_params g, int32_t* prompt_len, int32_t* output_len,
                                                      float* srv_ttft, float* srv_tbt, float* dev_pre_spt,
                                                      float* dev_dec_spt)
{
    i64 i = (i64)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= g.n_req) return;
    Words w = philox4x32_10(g.seed, (u64)i, F_PROMPT);
    prompt_len[i] = floor_clamp(gen_lognormal(w.w0, w.w1, g.prompt_mu, g.prompt_sigma), g.prompt_lo, g.prompt_hi);
    w = philox4x32_10(g.seed, (u64)i, F_OUTPUT);
    output_len[i] = floor_clamp(gen_lognormal(w.w0, w.w1, g.out_mu, g.out_sigma), g.out_lo, g.out_hi);
    w = philox4x32_10(g.seed, (u64)i, F_TTFT);
    float s;
    if (u23(w.w2) < g.ttft_pareto_p) {
        float inv_alpha = __fdiv_rn(1.0f, g.ttft_pareto_alpha);
        float e = -gen_ln(u23(w.w3));
        e = e * inv_alpha;
        s = g.ttft_pareto_xm * gen_exp(e);
    } else {
        s = gen_lognormal(w.w0, w.w1, g.ttft_mu, g.ttft_sigma);
    }
    srv_ttft[i] = s;
    w = philox4x32_10(g.seed, (u64)i, F_TBT);
    srv_tbt[i] = gen_lognormal(w.w0, w.w1, g.tbt_mu, g.tbt_sigma);
    w = philox4x32_10(g.seed, (u64)i, F_DEVICE);
    float dec, pre;
    if (g.dev_mode == 0) {
        dec = g.dev_a; pre = g.dev_b;
    } else {
        float rate;
        if (g.dev_mode == 1) rate = __fmaf_rn(u23(w.w0), g.dev_b - g.dev_a, g.dev_a);
        else rate = (u23(w.w0) < g.dev_p) ? g.dev_a : g.dev_b;
        dec = __fdiv_rn(1.0f, rate);
        pre = __fdiv_rn(dec, g.dev_pre_ratio);
    }
    dev_dec_spt[i] = dec;
    dev_pre_spt[i] = pre;
}

// Exclusive prefix sum of output_len into tok_off[0..n] in two launches: the sum of every tile, then per tile the
// sum of the tiles in front of it and a scan of its own elements.  Integer sums: any order gives the same offsets.
constexpr int GO_BLOCK = 1024;
constexpr int GO_MAX_TILES = 65536;
// Tile sums between the two launches (device memory of the library's code object, referenced by device code only).
// Calls of disco_gen_trace on one GPU share it: they must not overlap in time.
__device__ i64 g_tile_sum[GO_MAX_TILES];

__device__ __forceinline__ i64 block_sum_1024(i64 v, i64* sh)
{
    for (int d = 32; d >= 1; d >>= 1) v += __shfl_xor(v, d, 64);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    __syncthreads();
    if (lane == 0) sh[wave] = v;
    __syncthreads();
    i64 t = 0;
    for (int w = 0; w < GO_BLOCK / 64; ++w) t += sh[w];
    return t;
}

__global__ __launch_bounds__(GO_BLOCK) void k_gen_tile_sums(i64 n, i64 per_thread, const int32_t* __restrict__ output_len)
{
    __shared__ i64 sh[GO_BLOCK / 64];
    const i64 tile = per_thread * GO_BLOCK;
    const i64 lo = (i64)blockIdx.x * tile;
    i64 acc = 0;
    for (i64 q = 0; q < per_thread; ++q) {                   // coalesced: consecutive threads, consecutive elements
        const i64 i = lo + q * GO_BLOCK + threadIdx.x;
        if (i < n) acc += output_len[i];
    }
    acc = block_sum_1024(acc, sh);
    if (threadIdx.x == 0) g_tile_sum[blockIdx.x] = acc;
}

__global__ __launch_bounds__(GO_BLOCK) void k_gen_offsets(i64 n, i64 per_thread, const int32_t* __restrict__ output_len,
                                                          i64* __restrict__ tok_off)
{
    __shared__ i64 sh[GO_BLOCK / 64];
    __shared__ i64 wsum[GO_BLOCK / 64];
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const i64 tile = per_thread * GO_BLOCK;
    const i64 lo = (i64)blockIdx.x * tile;
    i64 before = 0;
    for (int b = threadIdx.x; b < (int)blockIdx.x; b += GO_BLOCK) before += g_tile_sum[b];
    i64 run = block_sum_1024(before, sh);                    // tokens of the tiles in front
    // the tile in rounds of 1024 consecutive elements: scan across the workgroup, carry `run`
    for (i64 q = 0; q < per_thread; ++q) {
        const i64 i = lo + q * GO_BLOCK + threadIdx.x;
        const i64 v = i < n ? (i64)output_len[i] : 0;
        i64 inc = v;
        for (int d = 1; d < 64; d <<= 1) {
            const i64 o = __shfl_up(inc, d, 64);
            if (lane >= d) inc += o;
        }
        __syncthreads();
        if (lane == 63) wsum[wave] = inc;
        __syncthreads();
        i64 front = 0, all = 0;
        for (int w = 0; w < GO_BLOCK / 64; ++w) { const i64 t = wsum[w]; front += w < wave ? t : 0; all += t; }
        if (i < n) tok_off[i] = run + front + inc - v;
        run += all;
    }
    if (blockIdx.x == gridDim.x - 1 && threadIdx.x == 0) tok_off[n] = run;
}

// Per-token gap in front of global token index j (the first token's is unused).
__global__ __launch_bounds__(256) void k_gen_gaps(disco_gen_params g, i64 n_tok, float* tok_arr)
{
    i64 j = (i64)blockIdx.x * blockDim.x + threadIdx.x;
    i64 stride = (i64)gridDim.x * blockDim.x;
    for (; j < n_tok; j += stride) {
        Words w = philox4x32_10(g.seed, (u64)j, F_GAP);
        float gap;
        if (u23(w.w2) < g.gap_stall_p)
            gap = __fmaf_rn(u23(w.w3), g.gap_stall_hi - g.gap_stall_lo, g.gap_stall_lo);
        else
            gap = gen_lognormal(w.w0, w.w1, g.gap_mu, g.gap_sigma);
        tok_arr[j] = gap;
    }
}

// Arrival offsets: running fp32 sum of a request's gaps in index order, in
// place.  The order of the additions is part of the trace's definition, so
// every request is summed by one thread, token after token; the tokens pass
// through LDS so that device memory is read and written in contiguous
// whole 128-byte lines: a workgroup takes 256 consecutive requests and moves
// one line (GA_K tokens) of each per round, 32 threads per request and line;
// the lines a request shares with its neighbours are touched by both, each
// moving only its own tokens.
constexpr int GA_BLOCK = 256;
constexpr int GA_K = 32;

__global__ __launch_bounds__(GA_BLOCK) void k_gen_arrivals(i64 n_req, const i64* __restrict__ tok_off, float* __restrict__ tok_arr)
{
    __shared__ float tile[GA_BLOCK][GA_K + 1];               // odd row stride: a thread per row without bank conflicts
    __shared__ i64 s_off[GA_BLOCK];                          // the 128-byte boundary at or below the request's first token
    __shared__ int s_lo[GA_BLOCK], s_len[GA_BLOCK];          // first token counted from that boundary, number of tokens
    __shared__ int s_max;
    const int t = threadIdx.x;
    const i64 i = (i64)blockIdx.x * GA_BLOCK + t;
    i64 a = 0;
    int lo = 0, len = 0;
    if (i < n_req) {
        const i64 first = tok_off[i];
        a = first & ~(i64)(GA_K - 1);                        // (tok_arr itself is at least 128-byte aligned)
        lo = (int)(first - a);
        len = (int)(tok_off[i + 1] - a);
    }
    if (t == 0) s_max = 0;
    s_off[t] = a; s_lo[t] = lo; s_len[t] = len - lo;
    __syncthreads();
    atomicMax(&s_max, len);
    __syncthreads();
    const int maxlen = s_max;
    const int sub = t & (GA_K - 1), grp = t / GA_K;
    float acc = 0.0f;
    for (int c0 = 0; c0 < maxlen; c0 += GA_K) {
        // pieces of GA_K tokens = whole 128-byte lines of the token array, 32 threads per request and piece
#pragma unroll 8
        for (int r = grp; r < GA_BLOCK; r += GA_BLOCK / GA_K)
            if ((unsigned)(c0 + sub - s_lo[r]) < (unsigned)s_len[r]) tile[r][sub] = tok_arr[s_off[r] + c0 + sub];
        __syncthreads();
        const int q0 = lo - c0 > 0 ? lo - c0 : 0, q1 = len - c0 < GA_K ? len - c0 : GA_K;
        for (int q = q0; q < q1; ++q) {
            if (c0 + q > lo) acc = acc + tile[t][q];         // (the first token's offset is 0, its gap unused)
            tile[t][q] = acc;
        }
        __syncthreads();
#pragma unroll 8
        for (int r = grp; r < GA_BLOCK; r += GA_BLOCK / GA_K)
            if ((unsigned)(c0 + sub - s_lo[r]) < (unsigned)s_len[r]) tok_arr[s_off[r] + c0 + sub] = tile[r][sub];
        __syncthreads();
    }
}

}  // namespace

extern "C" int32_t disco_gen_trace(const disco_gen_params* g, disco_trace* tr, int32_t stages, void* stream_)
{
    if (!g || !tr) return DISCO_ERR_NULL;
    hipStream_t stream = (hipStream_t)stream_;
    if (g->n_req < 0 || tr->n_req != g->n_req) return DISCO_ERR_SHAPE;
    if (g->prompt_lo > g->prompt_hi || g->out_lo > g->out_hi || g->out_lo < 1 || g->prompt_lo < 0) return DISCO_ERR_SHAPE;
    if (!(stages & (DISCO_GEN_REQUESTS | DISCO_GEN_TOKENS))) return DISCO_ERR_RANGE;
    auto prob = [](float p) { return p >= 0.0f && p <= 1.0f; };
    if (!(g->prompt_sigma >= 0) || !(g->out_sigma >= 0) || !(g->ttft_sigma >= 0) || !(g->tbt_sigma >= 0) ||
        !(g->gap_sigma >= 0) || !prob(g->ttft_pareto_p) || !prob(g->gap_stall_p) || !prob(g->dev_p) ||
        !(g->ttft_pareto_alpha > 0) || !(g->ttft_pareto_xm > 0) || g->dev_mode < 0 || g->dev_mode > 2 ||
        !(g->dev_a > 0) || !(g->dev_b > 0) || (g->dev_mode != 0 && !(g->dev_pre_ratio > 0)) ||
        (g->dev_mode == 1 && g->dev_b < g->dev_a) || g->gap_stall_hi < g->gap_stall_lo || g->gap_stall_lo < 0)
        return DISCO_ERR_RANGE;
    const i64 n = g->n_req;
    if (stages & DISCO_GEN_REQUESTS) {
        if (!tr->tok_off) return DISCO_ERR_NULL;
        if (n > 0 && (!tr->prompt_len || !tr->output_len || !tr->srv_ttft || !tr->srv_tbt || !tr->dev_pre_spt ||
                      !tr->dev_dec_spt))
            return DISCO_ERR_NULL;
        if (n > 0) {
            unsigned blocks = (unsigned)((n + 255) / 256);
            hipLaunchKernelGGL(k_gen_requests, dim3(blocks), dim3(256), 0, stream, *g, tr->prompt_len, tr->output_len,
                               tr->srv_ttft, tr->srv_tbt, tr->dev_pre_spt, tr->dev_dec_spt);
        }
        {
            i64 per_thread = 4;                              // tiles of 4096 requests while the tile sums fit
            while ((n + per_thread * GO_BLOCK - 1) / (per_thread * GO_BLOCK) > GO_MAX_TILES) per_thread *= 2;
            i64 tiles = (n + per_thread * GO_BLOCK - 1) / (per_thread * GO_BLOCK);
            if (tiles < 1) tiles = 1;
            hipLaunchKernelGGL(k_gen_tile_sums, dim3((unsigned)tiles), dim3(GO_BLOCK), 0, stream, n, per_thread, tr->output_len);
            hipLaunchKernelGGL(k_gen_offsets, dim3((unsigned)tiles), dim3(GO_BLOCK), 0, stream, n, per_thread, tr->output_len,
                               tr->tok_off);
        }
        DISCO_HIP(hipGetLastError());
        i64 total = 0;
        DISCO_HIP(hipMemcpyAsync(&total, tr->tok_off + n, sizeof(i64), hipMemcpyDeviceToHost, stream));
        DISCO_HIP(hipStreamSynchronize(stream));
        tr->n_tok = total;
    }
    if (stages & DISCO_GEN_TOKENS) {
        if (tr->n_tok < 0) return DISCO_ERR_SHAPE;
        if (tr->n_tok > 0) {
            if (!tr->tok_arr || !tr->tok_off) return DISCO_ERR_NULL;
            i64 want = (tr->n_tok + 255) / 256;
            unsigned blocks = (unsigned)(want < 65536 ? want : 65536);
            hipLaunchKernelGGL(k_gen_gaps, dim3(blocks), dim3(256), 0, stream, *g, tr->n_tok, tr->tok_arr);
            hipLaunchKernelGGL(k_gen_arrivals, dim3((unsigned)((n + GA_BLOCK - 1) / GA_BLOCK)), dim3(GA_BLOCK), 0, stream, n,
                               tr->tok_off, tr->tok_arr);
            DISCO_HIP(hipGetLastError());
        }
    }
    return DISCO_OK;
}
