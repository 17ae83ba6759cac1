/*
 * disco_oracle.c -- plain, slow, sequential CPU statement of what the DiSCo
 * evaluation path computes.  TEST INFRASTRUCTURE ONLY: it exists so that the
 * GPU library can be checked against it.  Nothing in the product path may
 * link, load or call this file; it shares no code, header, table or constant
 * generator with the GPU library.
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -shared -fPIC (no SIMD
 * intrinsics, no threads, no blocking or fusion).
 *
 * Every function below names the passage of the DiSCo paper (arXiv 2502.11417)
 * it follows.  Where the paper leaves a detail open the choice made is spelled
 * out in the comment of the function that makes it.
 *
 * Precision: the method is evaluated in fp32 for times (so that decisions,
 * migration indices and selected order statistics are decided in the same
 * precision as the library under test), exact int64 for token counts and fp64
 * for sums and costs.  fp32 expressions are written one IEEE operation at a
 * time; fused multiply-adds are explicit fmaf() calls and the compiler is
 * told not to contract.
 *
 * Pins (tests that do not go through this file's own formulas):
 *   philox            known-answer vectors of the generator's publication
 *   ln/exp/cos2pi     libm in fp64
 *   samplers          closed-form moments/quantiles of the distributions
 *   dispatch          zero budget / full budget / long wait special cases
 *   max-plus pacing   O(n^2) brute force in exact rational arithmetic
 *   LAG migration     constructed single-stall cases + closed-form tail
 *   buffer migration  constant-gap closed forms (hand-off index, delayed tokens), sequential
 *                     buffer simulation in exact rational arithmetic, cost-condition breakpoints
 *   quantile          numpy sort + nearest rank
 *   budget search     sort + prefix-sum solve; breakpoint enumeration (wait and ramp slope, the latter against
 *                     Eq. 2's sum written out)
 *   stochastic        zero / full budget equal the single-endpoint columns, binomial routing
 *                     frequency and token share, nesting in the budget, independence of runs,
 *                     the draw rebuilt from the pinned generator with counter and key spelled out
 * parity unpinned (conventions the paper does not fix; both sides follow the
 * same written reading): exchange rate lambda, pacing interval, budget-level
 * grid, tie-breaks, charging of a terminated loser, migration overhead time,
 * definition of "server lag", arrival process of the target after a buffer hand-off.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------ */
/* Counter-based generator: Philox4x32-10 (Salmon, Moraes, Dror, Shaw,       */
/* "Parallel Random Numbers: As Easy as 1, 2, 3", SC'11).                    */
/* ------------------------------------------------------------------------ */

void orc_philox_raw(const uint32_t ctr[4], const uint32_t key[2], uint32_t out[4])
{
    uint32_t c0 = ctr[0], c1 = ctr[1], c2 = ctr[2], c3 = ctr[3];
    uint32_t k0 = key[0], k1 = key[1];
    for (int round = 0; round < 10; ++round) {
        uint64_t prod_a = (uint64_t)0xD2511F53u * (uint64_t)c0;
        uint64_t prod_b = (uint64_t)0xCD9E8D57u * (uint64_t)c2;
        uint32_t n0 = (uint32_t)(prod_b >> 32) ^ c1 ^ k0;
        uint32_t n1 = (uint32_t)prod_b;
        uint32_t n2 = (uint32_t)(prod_a >> 32) ^ c3 ^ k1;
        uint32_t n3 = (uint32_t)prod_a;
        c0 = n0; c1 = n1; c2 = n2; c3 = n3;
        k0 += 0x9E3779B9u;   /* Weyl sequence, golden ratio */
        k1 += 0xBB67AE85u;   /* Weyl sequence, sqrt(3)-1    */
    }
    out[0] = c0; out[1] = c1; out[2] = c2; out[3] = c3;
}

/* Element `index` of random field `field` under `seed`:
 * key = seed, counter = (index_lo, index_hi, field, 0).  Every element is
 * independent of how elements are mapped to threads. */
void orc_philox(uint64_t seed, uint64_t index, uint32_t field, uint32_t out[4])
{
    uint32_t ctr[4] = { (uint32_t)index, (uint32_t)(index >> 32), field, 0u };
    uint32_t key[2] = { (uint32_t)seed, (uint32_t)(seed >> 32) };
    orc_philox_raw(ctr, key, out);
}

/* 23 random bits -> uniform on the open interval (0,1), exactly representable:
 * U = (floor(x / 2^9) + 1/2) * 2^-23. */
float orc_u23(uint32_t x)
{
    return fmaf((float)(x >> 9), 0x1p-23f, 0x1p-24f);
}

/* ------------------------------------------------------------------------ */
/* Elementary functions of the generator, defined as fixed sequences of IEEE */
/* fp32 operations so that every implementation returns the same bits.       */
/* ------------------------------------------------------------------------ */

static uint32_t f2u(float x) { uint32_t u; memcpy(&u, &x, 4); return u; }
static float u2f(uint32_t u) { float x; memcpy(&x, &u, 4); return x; }

/* Natural logarithm of a positive normal fp32 number.
 * x = 2^e * m, m in (sqrt(1/2), sqrt(2)]; ln m = 2 atanh(s), s = (m-1)/(m+1),
 * odd Taylor series through s^11. */
float orc_ln(float x)
{
    uint32_t bits = f2u(x);
    int32_t e = (int32_t)(bits >> 23) - 127;
    float m = u2f((bits & 0x007FFFFFu) | 0x3F800000u);
    if (m > 1.41421354f) { m = m * 0.5f; e = e + 1; }
    float f = m - 1.0f;
    float s = f / (2.0f + f);
    float z = s * s;
    float p = fmaf(z, 0.181818187f, 0.222222224f);   /* 2/11, 2/9 */
    p = fmaf(z, p, 0.285714298f);                     /* 2/7 */
    p = fmaf(z, p, 0.400000006f);                     /* 2/5 */
    p = fmaf(z, p, 0.666666687f);                     /* 2/3 */
    float sz = s * z;
    float lnm = fmaf(sz, p, 2.0f * s);
    return fmaf((float)e, 0.693147182f, lnm);
}

/* Exponential: clamp to [-86, 88], x = n ln2 + r with n = rint(x log2 e),
 * Taylor series of e^r through r^7, exact scaling by 2^n. */
float orc_exp(float x)
{
    if (x < -86.0f) x = -86.0f;
    if (x > 88.0f) x = 88.0f;
    float t = x * 1.44269502f;
    float n = rintf(t);
    float r = fmaf(n, -0.693145752f, x);        /* ln2 high part, 0x3f317200 */
    r = fmaf(n, -1.42860677e-06f, r);           /* ln2 low part */
    float p = fmaf(r, 1.98412701e-04f, 1.38888892e-03f);   /* 1/5040, 1/720 */
    p = fmaf(r, p, 8.33333377e-03f);            /* 1/120 */
    p = fmaf(r, p, 4.16666679e-02f);            /* 1/24 */
    p = fmaf(r, p, 0.166666672f);               /* 1/6 */
    p = fmaf(r, p, 0.5f);
    p = fmaf(r, p, 1.0f);
    p = fmaf(r, p, 1.0f);
    int32_t ni = (int32_t)n;
    float scale = u2f((uint32_t)(ni + 127) << 23);
    return p * scale;
}

/* cos(2 pi u) for u in (0,1): quadrant q = rint(4u), v = u - q/4 (exact),
 * a = 2 pi v in [-pi/4, pi/4], Taylor series of sin/cos. */
float orc_cos2pi(float u)
{
    float q = rintf(4.0f * u);
    float v = fmaf(q, -0.25f, u);
    float a = v * 6.28318548f;
    float a2 = a * a;
    float c = fmaf(a2, -2.75573200e-07f, 2.48015876e-05f);  /* -1/10!, 1/8! */
    c = fmaf(a2, c, -1.38888892e-03f);                       /* -1/6! */
    c = fmaf(a2, c, 4.16666679e-02f);                        /* 1/4! */
    c = fmaf(a2, c, -0.5f);
    c = fmaf(a2, c, 1.0f);
    float s = fmaf(a2, -2.50521079e-08f, 2.75573188e-06f);  /* -1/11!, 1/9! */
    s = fmaf(a2, s, -1.98412701e-04f);                       /* -1/7! */
    s = fmaf(a2, s, 8.33333377e-03f);                        /* 1/5! */
    s = fmaf(a2, s, -0.166666672f);                          /* -1/3! */
    s = fmaf(a2, s, 1.0f);
    s = s * a;
    int32_t qi = (int32_t)q & 3;
    if (qi == 0) return c;
    if (qi == 1) return -s;
    if (qi == 2) return -c;
    return s;
}

/* Standard normal by the Box-Muller transform of two uniforms. */
float orc_normal(uint32_t w0, uint32_t w1)
{
    float rad = sqrtf(-2.0f * orc_ln(orc_u23(w0)));
    return rad * orc_cos2pi(orc_u23(w1));
}

float orc_lognormal(uint32_t w0, uint32_t w1, float mu, float sigma)
{
    return orc_exp(fmaf(sigma, orc_normal(w0, w1), mu));
}

static int32_t floor_clamp(float v, int32_t lo, int32_t hi)
{
    float f = floorf(v);
    if (f < (float)lo) f = (float)lo;
    if (f > (float)hi) f = (float)hi;
    return (int32_t)f;
}

/* ------------------------------------------------------------------------ */
/* Synthetic trace (stand-in for the server traces and device profiles of    */
/* Sec. 5.1).  Precedent: the scalability study of Sec. 5.3 fits log-normal  */
/* laws to prompt length and server TTFT; server TTFT is independent of      */
/* prompt length (Sec. 3, Pearson table); device TTFT is linear in it.       */
/* ------------------------------------------------------------------------ */

typedef struct orc_gen_cfg {
    uint64_t seed;
    int64_t n_req;
    float prompt_mu, prompt_sigma; int32_t prompt_lo, prompt_hi;
    float out_mu, out_sigma; int32_t out_lo, out_hi;
    /* server TTFT: with probability pareto_p a Pareto(xm, alpha) draw,
     * otherwise log-normal(mu, sigma) */
    float ttft_mu, ttft_sigma, ttft_pareto_p, ttft_pareto_xm, ttft_pareto_alpha;
    float tbt_mu, tbt_sigma;            /* per-request constant server gap */
    /* device decode speed: 0 constant (dev_a = s/token decode, dev_b = s/token
     * prefill), 1 uniform on [dev_a, dev_b] tokens/s, 2 two-point: dev_a
     * tokens/s with probability dev_p else dev_b tokens/s.  In modes 1 and 2
     * prefill is dev_pre_ratio times faster than decode. */
    int32_t dev_mode; float dev_a, dev_b, dev_p, dev_pre_ratio;
    /* per-token server gaps: log-normal, replaced with probability stall_p by
     * a stall uniform on [stall_lo, stall_hi] seconds */
    float gap_mu, gap_sigma, gap_stall_p, gap_stall_lo, gap_stall_hi;
} orc_gen_cfg;

enum { F_PROMPT = 0, F_OUTPUT = 1, F_TTFT = 2, F_TBT = 3, F_DEVICE = 4, F_GAP = 5, F_ROUTE = 6 };

/* Per-request fields and the CSR offsets of the token array. */
void orc_gen_requests(const orc_gen_cfg* g, int32_t* prompt_len, int32_t* output_len,
                      float* srv_ttft, float* srv_tbt, float* dev_pre_spt,
                      float* dev_dec_spt, int64_t* tok_off)
{
    uint32_t w[4];
    int64_t running = 0;
    for (int64_t i = 0; i < g->n_req; ++i) {
        orc_philox(g->seed, (uint64_t)i, F_PROMPT, w);
        prompt_len[i] = floor_clamp(orc_lognormal(w[0], w[1], g->prompt_mu, g->prompt_sigma),
                                    g->prompt_lo, g->prompt_hi);
        orc_philox(g->seed, (uint64_t)i, F_OUTPUT, w);
        output_len[i] = floor_clamp(orc_lognormal(w[0], w[1], g->out_mu, g->out_sigma),
                                    g->out_lo, g->out_hi);
        orc_philox(g->seed, (uint64_t)i, F_TTFT, w);
        if (orc_u23(w[2]) < g->ttft_pareto_p) {
            float inv_alpha = 1.0f / g->ttft_pareto_alpha;
            float e = -orc_ln(orc_u23(w[3]));
            e = e * inv_alpha;
            srv_ttft[i] = g->ttft_pareto_xm * orc_exp(e);
        } else {
            srv_ttft[i] = orc_lognormal(w[0], w[1], g->ttft_mu, g->ttft_sigma);
        }
        orc_philox(g->seed, (uint64_t)i, F_TBT, w);
        srv_tbt[i] = orc_lognormal(w[0], w[1], g->tbt_mu, g->tbt_sigma);
        orc_philox(g->seed, (uint64_t)i, F_DEVICE, w);
        float dec, pre;
        if (g->dev_mode == 0) {
            dec = g->dev_a; pre = g->dev_b;
        } else {
            float rate;
            if (g->dev_mode == 1) rate = fmaf(orc_u23(w[0]), g->dev_b - g->dev_a, g->dev_a);
            else rate = (orc_u23(w[0]) < g->dev_p) ? g->dev_a : g->dev_b;
            dec = 1.0f / rate;
            pre = dec / g->dev_pre_ratio;
        }
        dev_dec_spt[i] = dec; dev_pre_spt[i] = pre;
        tok_off[i] = running;
        running += output_len[i];
    }
    tok_off[g->n_req] = running;
}

/* Gap in front of global token index `j` (field F_GAP). */
float orc_gen_gap(const orc_gen_cfg* g, int64_t j)
{
    uint32_t w[4];
    orc_philox(g->seed, (uint64_t)j, F_GAP, w);
    if (orc_u23(w[2]) < g->gap_stall_p)
        return fmaf(orc_u23(w[3]), g->gap_stall_hi - g->gap_stall_lo, g->gap_stall_lo);
    return orc_lognormal(w[0], w[1], g->gap_mu, g->gap_sigma);
}

/* Server arrival offsets of requests [req_lo, req_hi): time since the
 * request's first token, a sequential fp32 running sum of its gaps in index
 * order.  `tok_arr` is indexed by global token index minus `base`. */
void orc_gen_tokens(const orc_gen_cfg* g, const int64_t* tok_off, int64_t req_lo,
                    int64_t req_hi, int64_t base, float* tok_arr)
{
    for (int64_t i = req_lo; i < req_hi; ++i) {
        float acc = 0.0f;
        for (int64_t j = tok_off[i]; j < tok_off[i + 1]; ++j) {
            if (j > tok_off[i]) acc = acc + orc_gen_gap(g, j);
            tok_arr[j - base] = acc;
        }
    }
}

/* ------------------------------------------------------------------------ */
/* Dispatch (Sec. 4.2; Alg. 2 device-constrained, Alg. 3 server-constrained) */
/* ------------------------------------------------------------------------ */

/* One policy column.  mode 0 = server-constrained length threshold (Alg. 3),
 * mode 1 = device-constrained wait time (Sec. 4.2 Eq. 1 and Alg. 2),
 * mode 2 / 3 = the stochastic baselines of Sec. 5.1 (Stoch-S / Stoch-D): each
 * request goes to one endpoint only, to the constrained one (server in mode
 * 2, device in mode 3) with probability beta = the budget ratio b, else to
 * the other; l_mid is the run number (independent draws per run; runs share
 * nothing, budget levels of one run share the draw and are therefore nested). */
typedef struct orc_policy {
    int32_t mode;
    int32_t l_th;
    int32_t l_mid;     /* Alg. 2: the one length given a partial wait; -1 none */
    float w_mid;
    float beta;        /* Eq. 1 slope; +inf turns the ramp into w_tail */
    float w_tail;      /* Phase-1 cap; +inf = never start the device */
    int32_t mig_mode;  /* 0 none, 1 lag-triggered hand-off to the device */
} orc_policy;

/* Device TTFT, linear in prompt length: T_d(l) = k l + c (Sec. 4.2). */
float orc_device_ttft(int32_t l, float k, float c)
{
    return fmaf((float)l, k, c);
}

/* Wait before the device starts (Eq. 1, united with the step form of
 * Alg. 2: zero up to l_th, one partial length l_mid, else min(beta l,
 * w_tail)). */
float orc_wait(const orc_policy* p, int32_t l)
{
    if (l <= p->l_th) return 0.0f;
    if (l == p->l_mid) return p->w_mid;
    float ramp = p->beta * (float)l;
    return (ramp < p->w_tail) ? ramp : p->w_tail;   /* NaN ramp -> w_tail */
}

/* Dispatch of one request under one policy.
 * decision: bit0 = server started, bit1 = device started, bit2 = device won.
 * Server-constrained (Alg. 3): l < l_th runs on the device alone; otherwise
 * both start at time 0 and the earlier first token wins.
 * Device-constrained (Sec. 4.2): the server starts at 0; the device starts
 * after w(l) only if the server has produced nothing by then (s > w, strict).
 * The endpoint with the earlier first token decodes; a tie goes to the
 * server. */
uint64_t orc_route_seed(int32_t run)
{
    return ((uint64_t)0x53544F43u << 32) | (uint64_t)(uint32_t)run;     /* high word: a tag no trace seed uses */
}

/* Uniform variate of request `i` in run `run` of the stochastic baselines:
 * word 0 of the generator at key = (run, tag), counter = (i_lo, i_hi, F_ROUTE, 0). */
float orc_route_uniform(int32_t run, int64_t i)
{
    uint32_t w[4];
    orc_philox(orc_route_seed(run), (uint64_t)i, F_ROUTE, w);
    return orc_u23(w[0]);
}

void orc_dispatch_one(const orc_policy* p, int32_t l, float s, float d, int64_t i,
                      uint8_t* decision, float* ttft)
{
    if (p->mode == 2 || p->mode == 3) {
        /* Stoch-S / Stoch-D (Sec. 5.1 baselines): random routing that meets the budget in expectation */
        int constrained = orc_route_uniform(p->l_mid, i) < p->beta;
        int to_server = (p->mode == 2) ? constrained : !constrained;
        if (to_server) { *decision = 1; *ttft = s; }
        else { *decision = 6; *ttft = d; }
        return;
    }
    if (p->mode == 0) {
        if (l < p->l_th) { *decision = 6; *ttft = d; return; }
        if (d < s) { *decision = 7; *ttft = d; }
        else { *decision = 3; *ttft = s; }
        return;
    }
    float w = orc_wait(p, l);
    if (!(s > w)) { *decision = 1; *ttft = s; return; }
    float x = w + d;
    if (x < s) { *decision = 7; *ttft = x; }
    else { *decision = 3; *ttft = s; }
}

/* All pairs.  Token accounting (budget definitions of Sec. 4.2; cost model of
 * Sec. 4.1 / App. E): every started endpoint is charged the whole prompt; the
 * winner is charged the n output tokens (the "w/o Migration" variant).
 * tok[j] = {S_pre, S_dec, D_pre, D_dec}; cnt[j] = {device started, device won}.
 * decision/ttft are [P][N], nullable. */
void orc_dispatch(int64_t N, int32_t P, const int32_t* prompt_len, const float* srv_ttft,
                  const int32_t* output_len, const float* dev_pre_spt, float dev_pre_spt_s,
                  float dev_ttft_c, const orc_policy* pol,
                  uint8_t* decision, float* ttft, int64_t* tok, double* ttft_sum, int64_t* cnt)
{
    for (int32_t j = 0; j < P; ++j) {
        int64_t s_pre = 0, s_dec = 0, d_pre = 0, d_dec = 0, started = 0, won = 0;
        double sum = 0.0;
        for (int64_t i = 0; i < N; ++i) {
            float k = dev_pre_spt ? dev_pre_spt[i] : dev_pre_spt_s;
            float d = orc_device_ttft(prompt_len[i], k, dev_ttft_c);
            uint8_t dec; float t;
            orc_dispatch_one(&pol[j], prompt_len[i], srv_ttft[i], d, i, &dec, &t);
            if (dec & 1) s_pre += prompt_len[i];
            if (dec & 2) { d_pre += prompt_len[i]; started += 1; }
            if (dec & 4) { d_dec += output_len[i]; won += 1; }
            else s_dec += output_len[i];
            sum += (double)t;
            if (decision) decision[(int64_t)j * N + i] = dec;
            if (ttft) ttft[(int64_t)j * N + i] = t;
        }
        tok[4 * j + 0] = s_pre; tok[4 * j + 1] = s_dec;
        tok[4 * j + 2] = d_pre; tok[4 * j + 3] = d_dec;
        cnt[2 * j + 0] = started; cnt[2 * j + 1] = won;
        ttft_sum[j] = sum;
    }
}

/* ------------------------------------------------------------------------ */
/* Paced delivery and migration (Sec. 4.3: token buffer consumed at the      */
/* user's rate; hand-off figure; lag trigger of the token-level workload).   */
/* ------------------------------------------------------------------------ */

/* Timeline of one request whose first token comes from `src_is_device`.
 * All times are relative to that first token.
 *   r_t       arrival offset of token t at the buffer (server: trace offsets,
 *             or t * gap when there is no per-token trace; device: t * g_dev)
 *   delta_t   delivery to the user: delta_0 = 0, delta_t = max(r_t,
 *             delta_{t-1} + tau), evaluated in the shifted domain
 *             u_t = r_t - t tau, M_t = max_{v<=t} u_v, delta_t = t tau + M_t
 *   lag_t     r_t - (delta_{t-1} + tau): how overdue token t is
 *   m         first t >= 1 with lag_t > kappa tau (server source, lag mode)
 * On a trigger the server stops; the device re-prefills the prompt plus the m
 * tokens already produced (only token ids move, no KV state: Sec. 4.3) and
 * generates tokens m..n-1:
 *   t_dec = (delta_{m-1} + tau) + kappa tau,  t_mig = k (l + m) + c,
 *   r'_t = t_dec + t_mig + (t - m + 1) g_dev          for t >= m.
 * Outputs: mig_idx (-1 none), t_last = delta_{n-1}; nullable delivered[n]
 * and tbt[n-1] (tbt[t-1] = delta_t - delta_{t-1}). */
void orc_timeline(int32_t n, const float* r_srv, float gap_const, int32_t src_is_device,
                  int32_t lag_mode, float tau, float kappa, int32_t l, float k, float c,
                  float g_dev, int32_t* mig_idx, float* t_last, float* delivered, float* tbt)
{
    float kt = kappa * tau;
    float M = 0.0f, prev = 0.0f, base = 0.0f;
    int32_t m = -1;
    for (int32_t t = 0; t < n; ++t) {
        float r;
        if (m >= 0) r = fmaf((float)(t - m + 1), g_dev, base);
        else if (src_is_device) r = (float)t * g_dev;
        else if (r_srv) r = r_srv[t];
        else r = (float)t * gap_const;
        if (m < 0 && lag_mode && !src_is_device && t >= 1) {
            float slot = prev + tau;
            float lag = r - slot;
            if (lag > kt) {
                m = t;
                float t_dec = slot + kt;
                float t_mig = fmaf((float)(l + m), k, c);
                base = t_dec + t_mig;
                r = fmaf((float)(t - m + 1), g_dev, base);
            }
        }
        float u = fmaf(-(float)t, tau, r);
        if (t == 0 || u > M) M = u;
        float del = fmaf((float)t, tau, M);
        if (delivered) delivered[t] = del;
        if (tbt && t >= 1) tbt[t - 1] = del - prev;
        prev = del;
    }
    *mig_idx = m;
    *t_last = prev;
}

/* Buffer-based, cost-triggered migration (Sec. 4.3, "Theoretical Migration
 * Framework" and "Buffer-Based Migration Protocol").  The constrained
 * endpoint produced the first token; decoding is handed to the other endpoint
 * as soon as (a) the buffer holds enough undelivered tokens to hide the
 * hand-off, B = r_c t_m tokens of playback, i.e. the playback time ahead of
 * the newest token covers the migration time:  delta_t - r_t >= t_mig(t)
 * (the rounding-free form of "buffer contains B tokens"), and (b) the decode
 * cost saved on the remaining tokens exceeds the overhead of prefilling the
 * target:  dc (n - 1 - t) > cp (l + t + 1)  (C_migration > Overhead).
 * The source stops after token m = the first such t; the target re-prefills
 * the prompt plus the m + 1 tokens produced so far (token ids only) and
 * delivers token m + 1 one gap after its prefill:
 *   t_mig(t)  device target: k (l + t + 1) + c;  server target: its TTFT s
 *   base      r_m + t_mig(m)
 *   r'_t      device: base + (t - m) g_dev;  server with a token trace:
 *             base + (r^S_t - r^S_m);  server with a constant gap:
 *             base + (t - m) gap_srv                            for t > m.
 * delay_num = number of tokens after the hand-off that reach the user late:
 * token t is late when it arrives after its pacing slot, r_t > delta_{t-1} +
 * tau (the buffer has run dry and the arrival, not the pacing, decides the
 * delivery; lag_t > 0 in the notation of orc_timeline).  In exact arithmetic
 * this is TBT_t > tau; stated on the arrival it does not depend on the
 * rounding of two paced deliveries, whose computed difference scatters by an
 * ulp around tau when tau is not a dyadic number.
 * Outputs: mig_last = m (-1 none), delay_num, t_last; nullable delivered, tbt. */
void orc_timeline_buffer(int32_t n, const float* r_srv, float gap_srv, int32_t src_is_device,
                         double dc, double cp, float srv_ttft, float tau, int32_t l, float k, float c,
                         float g_dev, int32_t* mig_last, int32_t* delay_num, float* t_last,
                         float* delivered, float* tbt)
{
    float M = 0.0f, prev = 0.0f, base = 0.0f, r_m = 0.0f;
    int32_t m = -1, delayed = 0;
    for (int32_t t = 0; t < n; ++t) {
        float r;
        if (m >= 0) {
            if (src_is_device) {                        /* target = server */
                if (r_srv) { float since = r_srv[t] - r_m; r = base + since; }
                else r = fmaf((float)(t - m), gap_srv, base);
            } else {
                r = fmaf((float)(t - m), g_dev, base);
            }
        } else if (src_is_device) r = (float)t * g_dev;
        else if (r_srv) r = r_srv[t];
        else r = (float)t * gap_srv;
        float u = fmaf(-(float)t, tau, r);
        if (t == 0 || u > M) M = u;
        float del = fmaf((float)t, tau, M);
        if (delivered) delivered[t] = del;
        if (t >= 1) {
            float gap = del - prev;
            if (tbt) tbt[t - 1] = gap;
            float slot = prev + tau;
            float lag = r - slot;
            if (m >= 0 && lag > 0.0f) delayed += 1;
        }
        if (m < 0 && t + 1 < n) {
            float slack = del - r;
            float t_mig = src_is_device ? srv_ttft : fmaf((float)(l + t + 1), k, c);
            double saved = dc * (double)(n - 1 - t);
            double overhead = cp * (double)(l + t + 1);
            if (slack >= t_mig && saved > overhead) {
                m = t;
                base = r + t_mig;
                r_m = (src_is_device && r_srv) ? r_srv[t] : 0.0f;
            }
        }
        prev = del;
    }
    *mig_last = m;
    *delay_num = delayed;
    *t_last = prev;
}

/* All pairs: each pair's source is the dispatch winner; timelines are
 * recomputed per pair (no sharing between columns).  mig_mode 1: lag hand-off
 * (server source).  mig_mode 2: buffer hand-off when the source is the
 * constrained endpoint of the column (modes 0, 2: server -> device, price
 * difference dc = cs_dec - lambda e_dec, target prefill price cp = lambda
 * e_pre; modes 1, 3: device -> server, dc = lambda e_dec - cs_dec, cp = cs_pre);
 * `rates` = {cs_pre, cs_dec, e_pre, e_dec, lambda} (needed for mode 2 only).
 * Per pair [P][N] (nullable): mig_idx (index of the first token produced by
 * the target, -1 none), n_src_tok (tokens produced by the source), t_last,
 * delay_num.  Per column: mtok[j] = {server decode tokens, device decode
 * tokens, device re-prefill tokens, server re-prefill tokens}, cnt[j] =
 * {migrated requests, number of TBT values, sum of delay_num}, tlast_sum[j].
 * If tbt_col >= 0 the TBT values of that column are written to tbt_out
 * (request order, token order), and delivered_out (indexed like the token
 * array) receives its delivery offsets. */
void orc_migration(int64_t N, int32_t P, const int32_t* prompt_len, const float* srv_ttft,
                   const int32_t* output_len, const float* srv_tbt,
                   const float* dev_pre_spt, float dev_pre_spt_s,
                   const float* dev_dec_spt, float dev_dec_spt_s, float dev_ttft_c,
                   const int64_t* tok_off, const float* tok_arr,
                   const orc_policy* pol, float tau, float kappa, const double* rates,
                   int32_t* mig_idx, int32_t* n_src_tok, float* t_last, int32_t* delay_num,
                   int64_t* mtok, int64_t* cnt, double* tlast_sum,
                   int32_t tbt_col, float* tbt_out, float* delivered_out)
{
    for (int32_t j = 0; j < P; ++j) {
        int64_t s_dec = 0, d_dec = 0, d_repre = 0, s_repre = 0, migrated = 0, n_tbt = 0, delay_sum = 0;
        double sum = 0.0;
        int64_t tbt_pos = 0, run_off = 0;
        for (int64_t i = 0; i < N; ++i) {
            float k = dev_pre_spt ? dev_pre_spt[i] : dev_pre_spt_s;
            float g = dev_dec_spt ? dev_dec_spt[i] : dev_dec_spt_s;
            int32_t l = prompt_len[i], n = output_len[i];
            float d = orc_device_ttft(l, k, dev_ttft_c);
            uint8_t dec; float ttft;
            orc_dispatch_one(&pol[j], l, srv_ttft[i], d, i, &dec, &ttft);
            int32_t src_dev = (dec & 4) ? 1 : 0;
            const float* r = (tok_arr && tok_off) ? tok_arr + tok_off[i] : NULL;
            int64_t off = tok_off ? tok_off[i] : run_off;
            int32_t m = -1, nsrc = n, delayed = 0; float tl;
            int want = (j == tbt_col);
            float* dl = (want && delivered_out) ? delivered_out + off : NULL;
            float* tb = (want && tbt_out) ? tbt_out + tbt_pos : NULL;
            float gap_srv = srv_tbt ? srv_tbt[i] : 0.0f;
            int buffer = pol[j].mig_mode == 2 && rates && (((pol[j].mode == 0 || pol[j].mode == 2) && !src_dev) || ((pol[j].mode == 1 || pol[j].mode == 3) && src_dev));
            if (buffer) {
                double dev_dec_price = rates[4] * rates[3], dev_pre_price = rates[4] * rates[2];
                double dc = src_dev ? dev_dec_price - rates[1] : rates[1] - dev_dec_price;
                double cp = src_dev ? rates[0] : dev_pre_price;
                int32_t last;
                orc_timeline_buffer(n, r, gap_srv, src_dev, dc, cp, srv_ttft[i], tau, l, k, dev_ttft_c, g,
                                    &last, &delayed, &tl, dl, tb);
                if (last >= 0) { m = last + 1; nsrc = last + 1; }
            } else {
                orc_timeline(n, r, gap_srv, src_dev, pol[j].mig_mode == 1, tau, kappa, l, k, dev_ttft_c, g,
                             &m, &tl, dl, tb);
                if (m >= 0) nsrc = m;
            }
            if (src_dev) { d_dec += nsrc; s_dec += n - nsrc; }
            else { s_dec += nsrc; d_dec += n - nsrc; }
            if (m >= 0) {
                migrated += 1;
                if (src_dev) s_repre += (int64_t)l + nsrc; else d_repre += (int64_t)l + nsrc;
                delay_sum += delayed;
            }
            n_tbt += n - 1;
            tbt_pos += n - 1;
            run_off += n;
            sum += (double)tl;
            if (mig_idx) mig_idx[(int64_t)j * N + i] = m;
            if (n_src_tok) n_src_tok[(int64_t)j * N + i] = nsrc;
            if (t_last) t_last[(int64_t)j * N + i] = tl;
            if (delay_num) delay_num[(int64_t)j * N + i] = delayed;
        }
        mtok[4 * j + 0] = s_dec; mtok[4 * j + 1] = d_dec; mtok[4 * j + 2] = d_repre; mtok[4 * j + 3] = s_repre;
        cnt[3 * j + 0] = migrated; cnt[3 * j + 1] = n_tbt; cnt[3 * j + 2] = delay_sum;
        tlast_sum[j] = sum;
    }
}

/* ------------------------------------------------------------------------ */
/* Unified cost (Sec. 4.1; App. E cost equation, read with separate prefill  */
/* and decode token counts per endpoint).                                    */
/* ------------------------------------------------------------------------ */

double orc_server_cost(double cs_pre, double cs_dec, int64_t s_pre, int64_t s_dec)
{
    return cs_pre * (double)s_pre + cs_dec * (double)s_dec;
}

double orc_device_energy(double e_pre, double e_dec, int64_t d_pre, int64_t d_dec)
{
    return e_pre * (double)d_pre + e_dec * (double)d_dec;
}

double orc_total_cost(double cs_pre, double cs_dec, double e_pre, double e_dec, double lambda,
                      int64_t s_pre, int64_t s_dec, int64_t d_pre, int64_t d_dec)
{
    double server = orc_server_cost(cs_pre, cs_dec, s_pre, s_dec);
    double energy = orc_device_energy(e_pre, e_dec, d_pre, d_dec);
    return server + lambda * energy;
}

/* ------------------------------------------------------------------------ */
/* Statistics (Sec. 5.1 metrics: mean and tail TTFT / TBT).                  */
/* ------------------------------------------------------------------------ */

static int cmp_float(const void* a, const void* b)
{
    float x = *(const float*)a, y = *(const float*)b;
    return (x > y) - (x < y);
}

/* Nearest-rank order statistic of M values: rank k = ceil(q M) (1-based,
 * q = num/den, clamped to [1, M]), value = k-th smallest.  Sorts a copy. */
int64_t orc_quantile(const float* v, int64_t M, int64_t num, int64_t den, float* value)
{
    if (M <= 0) { *value = NAN; return 0; }
    int64_t k = (num * M + den - 1) / den;
    if (k < 1) k = 1;
    if (k > M) k = M;
    float* tmp = (float*)malloc((size_t)M * sizeof(float));
    memcpy(tmp, v, (size_t)M * sizeof(float));
    qsort(tmp, (size_t)M, sizeof(float), cmp_float);
    *value = tmp[k - 1];
    free(tmp);
    return k;
}

/* ------------------------------------------------------------------------ */
/* Budget search.                                                            */
/* ------------------------------------------------------------------------ */

enum { ACC_TOTAL_COST = 0, ACC_SERVER_COST = 1, ACC_DEVICE_COST = 2,
       ACC_SERVER_PREFILL_TOK = 3, ACC_DEVICE_PREFILL_TOK = 4 };

static double accumulator(int32_t which, const double* rates /* cs_pre, cs_dec, e_pre, e_dec, lambda */,
                          const int64_t* tok)
{
    switch (which) {
    case ACC_TOTAL_COST:
        return orc_total_cost(rates[0], rates[1], rates[2], rates[3], rates[4],
                              tok[0], tok[1], tok[2], tok[3]);
    case ACC_SERVER_COST: return orc_server_cost(rates[0], rates[1], tok[0], tok[1]);
    case ACC_DEVICE_COST: return rates[4] * orc_device_energy(rates[2], rates[3], tok[2], tok[3]);
    case ACC_SERVER_PREFILL_TOK: return (double)tok[0];
    default: return (double)tok[2];
    }
}

static double eval_acc(int64_t N, const int32_t* prompt_len, const float* srv_ttft,
                       const int32_t* output_len, const float* dev_pre_spt, float dev_pre_spt_s,
                       float dev_ttft_c, const orc_policy* p, int32_t which, const double* rates)
{
    int64_t tok[4], cnt[2]; double sum;
    orc_dispatch(N, 1, prompt_len, srv_ttft, output_len, dev_pre_spt, dev_pre_spt_s,
                 dev_ttft_c, p, NULL, NULL, tok, &sum, cnt);
    return accumulator(which, rates, tok);
}

/* Bisection on the wait cap w_tail of a device-constrained policy so that an
 * accumulator that does not increase with the wait meets `target` (the
 * budget of Sec. 4.2 is an allowance for the constrained endpoint; Alg. 2
 * asks for the wait that meets it).  fp32 midpoints; the accumulator comes
 * from exact token totals.  A(mid) > target moves lo up, else hi down; the
 * answer is hi (the side that respects the budget).  hist_*[n_steps]. */
float orc_search_wait(int64_t N, const int32_t* prompt_len, const float* srv_ttft,
                      const int32_t* output_len, const float* dev_pre_spt, float dev_pre_spt_s,
                      float dev_ttft_c, const orc_policy* templ, float lo, float hi,
                      int32_t n_steps, int32_t which, const double* rates, double target,
                      float* hist_param, double* hist_acc)
{
    orc_policy p = *templ;
    for (int32_t step = 0; step < n_steps; ++step) {
        float mid = 0.5f * (lo + hi);
        p.w_tail = mid;
        double a = eval_acc(N, prompt_len, srv_ttft, output_len, dev_pre_spt, dev_pre_spt_s,
                            dev_ttft_c, &p, which, rates);
        hist_param[step] = mid; hist_acc[step] = a;
        if (a > target) lo = mid; else hi = mid;
    }
    return hi;
}

/* Bisection on the slope beta of the ramp w(l) = min(beta l, w_tail) of Eq. 1 for the prompts above l_th, so that
 * an accumulator that does not increase with the slope meets `target`: Eq. 2 asks for the beta at which the device
 * prefill of those prompts uses up what is left of the budget.  Here the left-hand side of Eq. 2 is taken on the
 * trace itself (every request starts the device iff its own server TTFT exceeds its wait), not on the product of
 * the two marginal distributions.  Same steps as orc_search_wait: fp32 midpoints, A(mid) > target moves lo up,
 * the answer is hi.  hist_*[n_steps]. */
float orc_search_slope(int64_t N, const int32_t* prompt_len, const float* srv_ttft,
                       const int32_t* output_len, const float* dev_pre_spt, float dev_pre_spt_s,
                       float dev_ttft_c, const orc_policy* templ, float lo, float hi,
                       int32_t n_steps, int32_t which, const double* rates, double target,
                       float* hist_param, double* hist_acc)
{
    orc_policy p = *templ;
    for (int32_t step = 0; step < n_steps; ++step) {
        float mid = 0.5f * (lo + hi);
        p.beta = mid;
        double a = eval_acc(N, prompt_len, srv_ttft, output_len, dev_pre_spt, dev_pre_spt_s,
                            dev_ttft_c, &p, which, rates);
        hist_param[step] = mid; hist_acc[step] = a;
        if (a > target) lo = mid; else hi = mid;
    }
    return hi;
}

/* Integer bisection on the length threshold of a server-constrained policy
 * (Eq. 3 in discrete form): the smallest l_th in [lo, hi] whose accumulator
 * (non-increasing in l_th, e.g. server prefill tokens) does not exceed
 * `target`; hi must satisfy it.  Steps after convergence re-evaluate at the
 * answer. */
int32_t orc_search_lth(int64_t N, const int32_t* prompt_len, const float* srv_ttft,
                       const int32_t* output_len, const float* dev_pre_spt, float dev_pre_spt_s,
                       float dev_ttft_c, const orc_policy* templ, int32_t lo, int32_t hi,
                       int32_t n_steps, int32_t which, const double* rates, double target,
                       int32_t* hist_param, double* hist_acc)
{
    orc_policy p = *templ;
    for (int32_t step = 0; step < n_steps; ++step) {
        int32_t mid = lo + (hi - lo) / 2;
        p.l_th = mid;
        double a = eval_acc(N, prompt_len, srv_ttft, output_len, dev_pre_spt, dev_pre_spt_s,
                            dev_ttft_c, &p, which, rates);
        hist_param[step] = mid; hist_acc[step] = a;
        if (lo < hi) { if (a > target) lo = mid + 1; else hi = mid; }
    }
    return hi;
}
