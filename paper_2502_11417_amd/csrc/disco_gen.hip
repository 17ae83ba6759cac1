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

// Exclusive prefix sum of output_len into tok_off[0..n], one workgroup: each
// thread owns a contiguous slice (sum, scan of the slice sums, write-out).
__global__ __launch_bounds__(1024) void k_gen_offsets(i64 n, const int32_t* output_len, i64* tok_off)
{
    __shared__ i64 sums[1024];
    const int t = threadIdx.x;
    i64 per = (n + 1023) / 1024;
    i64 a = (i64)t * per, b = a + per;
    if (a > n) a = n;
    if (b > n) b = n;
    i64 acc = 0;
    for (i64 i = a; i < b; ++i) acc += output_len[i];
    sums[t] = acc;
    __syncthreads();
    for (int d = 1; d < 1024; d <<= 1) {
        i64 v = (t >= d) ? sums[t - d] : 0;
        __syncthreads();
        sums[t] += v;
        __syncthreads();
    }
    i64 run = (t == 0) ? 0 : sums[t - 1];
    for (i64 i = a; i < b; ++i) { tok_off[i] = run; run += output_len[i]; }
    if (t == 1023) tok_off[n] = sums[1023];
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
// place, one request per thread (the order of the additions is part of the
// trace's definition, so this step is sequential per request).
__global__ __launch_bounds__(256) void k_gen_arrivals(i64 n_req, const i64* tok_off, float* tok_arr)
{
    i64 i = (i64)blockIdx.x * blockDim.x + threadIdx.x;
    if (i >= n_req) return;
    i64 a = tok_off[i], b = tok_off[i + 1];
    float acc = 0.0f;
    for (i64 j = a; j < b; ++j) {
        if (j > a) acc = acc + tok_arr[j];
        tok_arr[j] = acc;
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
        hipLaunchKernelGGL(k_gen_offsets, dim3(1), dim3(1024), 0, stream, n, tr->output_len, tr->tok_off);
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
            hipLaunchKernelGGL(k_gen_arrivals, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, stream, n, tr->tok_off,
                               tr->tok_arr);
            DISCO_HIP(hipGetLastError());
        }
    }
    return DISCO_OK;
}
