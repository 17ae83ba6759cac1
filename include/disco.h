/*
 * disco.h -- C ABI of libdisco: batched, trace-driven evaluation of the DiSCo
 * device/server dispatch and token-level migration policies (arXiv 2502.11417)
 * over (request x policy-column) pairs on one AMD MI355X (gfx950).
 *
 * Conventions that hold for every entry point
 * -------------------------------------------
 *  - "host" pointers are ordinary process memory, read during the call only.
 *    "device" pointers are HIP device memory that the caller allocated, owns
 *    and keeps alive until the work enqueued by the call has finished.  The
 *    library never allocates, frees or retains device memory.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    All work is enqueued on it and the calls return without waiting, except
 *    where a call says it synchronises.  The asynchronous calls enqueue kernel
 *    launches only (no memset or copy operations), so a sequence of them can
 *    be captured into a HIP graph on a capturing stream and replayed.
 *  - Policy tables (`pol`, `templ`) may live in host or in device memory; the
 *    library asks the HIP runtime which it is.  A host table is validated
 *    (DISCO_ERR_RANGE for unknown modes or NaN parameters); a device table,
 *    e.g. the pol_out of disco_budget_search, is used as it is, which keeps a
 *    search -> evaluate -> reduce sequence free of host round trips.
 *  - Return value: DISCO_OK or a negative DISCO_ERR_* code.  Shapes, null
 *    pointers and workspace sizes are checked on the host before anything is
 *    launched; a failed check launches nothing.  No exceptions, no abort.
 *  - Times are fp32 seconds, lengths int32 tokens, CSR offsets int64, token
 *    totals int64, sums and costs fp64.
 *  - Per-pair arrays are policy-major: element (column j, request i) is at
 *    [j * n_req + i].
 */
#ifndef DISCO_H
#define DISCO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define DISCO_OK              0
#define DISCO_ERR_NULL      (-1)  /* a required pointer is NULL */
#define DISCO_ERR_SHAPE     (-2)  /* negative or inconsistent sizes, P outside [1, DISCO_MAX_COLS] */
#define DISCO_ERR_RANGE     (-3)  /* a parameter (or, disco_validate_trace, a trace value) outside its documented range */
#define DISCO_ERR_CSR       (-4)  /* token arrays required by the call are missing (disco_validate_trace: inconsistent) */
#define DISCO_ERR_WORKSPACE (-5)  /* workspace missing or smaller than disco_workspace_bytes() */
#define DISCO_ERR_HIP       (-6)  /* a HIP runtime call failed; see disco_last_hip_error() */

#define DISCO_MAX_COLS   64       /* policy columns per call */
#define DISCO_MAX_Q       4       /* quantiles per call */
#define DISCO_MAX_STEPS  64       /* bisection steps per search */

/* ---- trace ------------------------------------------------------------- */

/* One batch of requests, structure-of-arrays, all arrays on the device.
 * The per-request measurements are the inputs the paper's policies assume to
 * be known (Sec. 4.2: the server TTFT distribution from profiling, the device
 * TTFT linear in prompt length, T_d(l) = k l + c).
 *   prompt_len[i]  l_i                       output_len[i]  n_i >= 1
 *   srv_ttft[i]    s_i > 0, server time to first token (network + queue + prefill)
 *   srv_tbt[i]     constant server gap, used only when tok_arr is NULL
 *   dev_pre_spt[i] k_i, device seconds per prompt token   (NULL: dev_pre_spt_s for all)
 *   dev_dec_spt[i] g_i, device seconds per decoded token  (NULL: dev_dec_spt_s for all)
 *   tok_off[n_req+1], tok_arr[n_tok]  CSR: server arrival offset of token t of
 *       request i, in seconds since that request's first token, at
 *       tok_arr[tok_off[i] + t]; tok_off[i+1] - tok_off[i] == output_len[i],
 *       tok_arr[tok_off[i]] == 0, non-decreasing inside a request.  Both NULL
 *       when the batch carries no per-token timeline.
 *   dev_ttft_c     c, the intercept of the device TTFT. */
typedef struct disco_trace {
    int64_t n_req;
    int64_t n_tok;
    int32_t* prompt_len;
    int32_t* output_len;
    float* srv_ttft;
    float* srv_tbt;
    float* dev_pre_spt;
    float* dev_dec_spt;
    int64_t* tok_off;
    float* tok_arr;
    float dev_pre_spt_s;
    float dev_dec_spt_s;
    float dev_ttft_c;
    float reserved;
} disco_trace;

/* Parameters of the synthetic trace that stands in for the measured server
 * traces and device profiles of Sec. 5.1 (recipe of the scalability study in
 * Sec. 5.3: log-normal prompt lengths and server TTFT; server TTFT independent
 * of prompt length, Sec. 3).  Element `index` of field f is a function of
 * (seed, f, index) alone: Philox4x32-10 with key = seed and counter =
 * (index_lo, index_hi, f, 0); f = 0 prompt_len, 1 output_len, 2 srv_ttft,
 * 3 srv_tbt, 4 device speed (index = request), 5 per-token gap (index =
 * global token index). */
typedef struct disco_gen_params {
    uint64_t seed;
    int64_t n_req;
    float prompt_mu, prompt_sigma; int32_t prompt_lo, prompt_hi;  /* l = clamp(floor(LN)) */
    float out_mu, out_sigma; int32_t out_lo, out_hi;              /* n = clamp(floor(LN)) */
    float ttft_mu, ttft_sigma;        /* s ~ LN(mu, sigma) with probability 1 - ttft_pareto_p */
    float ttft_pareto_p, ttft_pareto_xm, ttft_pareto_alpha;       /* else Pareto(xm, alpha) */
    float tbt_mu, tbt_sigma;          /* per-request constant server gap ~ LN */
    int32_t dev_mode;                 /* 0: g = dev_a s/token, k = dev_b s/token;
                                         1: decode rate uniform on [dev_a, dev_b] tokens/s;
                                         2: rate dev_a tokens/s with probability dev_p, else dev_b;
                                         modes 1, 2: k = g / dev_pre_ratio */
    float dev_a, dev_b, dev_p, dev_pre_ratio;
    float gap_mu, gap_sigma;          /* per-token server gap ~ LN, replaced with probability */
    float gap_stall_p, gap_stall_lo, gap_stall_hi;   /* gap_stall_p by U[lo, hi] seconds */
} disco_gen_params;

#define DISCO_GEN_REQUESTS 1   /* per-request arrays and tok_off */
#define DISCO_GEN_TOKENS   2   /* tok_arr from tok_off (after DISCO_GEN_REQUESTS) */

/* Fill a trace on the device.  `trace` is a host struct whose device arrays
 * the caller allocated: n_req elements each (tok_off: n_req + 1; every
 * per-request array including dev_pre_spt / dev_dec_spt is required).
 * stages & DISCO_GEN_REQUESTS: writes the per-request arrays and tok_off,
 *   then SYNCHRONISES the stream and stores the token total in trace->n_tok
 *   so that the caller can size tok_arr.
 * stages & DISCO_GEN_TOKENS: writes tok_arr[0 .. trace->n_tok) (asynchronous);
 *   trace->n_tok must equal tok_off[n_req].  The arrival offsets of a request
 *   are the running fp32 sum, in index order, of its per-token gaps.
 * Calls on one GPU share a small area of device memory inside the library
 * (tile sums of the offset scan): do not let two of them overlap in time.
 * Errors: NULL (struct or a required array), SHAPE (n_req < 0, lo > hi),
 * RANGE (sigma < 0, probabilities outside [0,1], rates <= 0), HIP. */
int32_t disco_gen_trace(const disco_gen_params* params /*host*/, disco_trace* trace /*host, device arrays*/,
                        int32_t stages, void* stream);

/* ---- recorded traces ---------------------------------------------------- */

/* A recorded trace (Sec. 5.1: the evaluation is driven by traces of production
 * services): wall-clock timestamps in seconds, fp64, device arrays.
 * t_send[i]: request i sent; t_token[tok_off[i] .. tok_off[i+1]): arrival of
 * each of its output tokens, in order. */
typedef struct disco_raw_trace {
    int64_t n_req, n_tok;
    const double* t_send;
    const double* t_token;
    const int64_t* tok_off;       /* [n_req + 1], tok_off[n_req] == n_tok */
} disco_raw_trace;

/* Fills the relative-time arrays of `trace` from `raw`: srv_ttft[i] = first
 * token's arrival - send time, tok_arr = arrival offsets since the request's
 * first token, output_len[i] = number of tokens; every difference is taken in
 * fp64 and rounded once to fp32.  trace->srv_ttft, output_len and tok_arr must
 * point to device arrays of n_req / n_req / n_tok elements; n_req, n_tok and
 * tok_off of `trace` are set from `raw` (the offsets are shared, not copied).
 * Prompt lengths and device speeds are the caller's (disco_device_profile).
 * A request without tokens gets output_len 0 and srv_ttft NaN and must be
 * dropped before evaluation.  Asynchronous.  Errors: NULL, SHAPE, HIP. */
int32_t disco_ingest_trace(const disco_raw_trace* raw /*host*/, disco_trace* trace /*host, device arrays*/, void* stream);

/* Optional check of a trace's data before it is evaluated (the evaluation calls
 * check pointers and sizes only and trust the arrays: offsets that do not
 * match the output lengths make them read outside the token array).  One pass
 * over the requests and, with check_tokens != 0 and a token array, one over
 * the tokens.  SYNCHRONISES the stream and returns
 *   DISCO_ERR_CSR    tok_off does not start at 0, decreases, does not end at
 *                    n_tok (with a token array), or tok_off[i+1] - tok_off[i]
 *                    != output_len[i];
 *   DISCO_ERR_RANGE  a prompt length < 0, an output length < 1, a NaN,
 *                    negative or infinite server TTFT, gap or device rate, or
 *                    (tokens) an arrival offset that is NaN, negative, not 0
 *                    for a request's first token or smaller than its predecessor;
 *   DISCO_OK         otherwise.
 * (A request without tokens, as disco_ingest_trace marks it, is a RANGE error:
 * drop it first.)  ws: device, at least 256 bytes, 256-byte aligned.
 * Other errors: NULL, SHAPE, WORKSPACE, HIP. */
int32_t disco_validate_trace(const disco_trace* trace /*host, device arrays*/, int32_t check_tokens,
                             void* ws /*device*/, size_t ws_bytes, void* stream);

/* Log-normal law fitted "by the mean and standard deviation of the logarithm"
 * (Sec. 5.3): mu = mean of ln x, sigma = population standard deviation of
 * ln x, over the positive values of x (the others are counted in n_skipped);
 * NaN when no value is positive.  They are the prompt_mu / prompt_sigma and
 * ttft_mu / ttft_sigma of disco_gen_params. */
typedef struct disco_lognormal_fit {
    double mu, sigma;
    int64_t n_used, n_skipped;
} disco_lognormal_fit;

#define DISCO_FIT_INT32   0   /* x is int32 (prompt lengths) */
#define DISCO_FIT_FLOAT32 1   /* x is fp32 (server TTFT) */

/* x: device, n values of the given kind; out: device.  fp64 arithmetic; two
 * passes (mean, then deviation), partial sums folded in a fixed order.
 * Asynchronous.  Errors: NULL, SHAPE (n < 0), RANGE (kind), WORKSPACE, HIP. */
int32_t disco_fit_lognormal(const void* x /*device*/, int32_t kind, int64_t n, disco_lognormal_fit* out /*device*/,
                            void* ws /*device*/, size_t ws_bytes, void* stream);

/* On-device configurations of the evaluation (Sec. 5.1), index 0..2: Pixel 7
 * Pro with Bloom 1.1B, Pixel 7 Pro with Bloom 560M, Xiaomi 14 with Qwen 1.5
 * 0.5B.  The seconds per token are the fp32 reciprocals of the printed
 * speeds and go into disco_trace.dev_pre_spt_s / dev_dec_spt_s; the device
 * TTFT is k l with no intercept.  Host only.  Errors: NULL, RANGE (index). */
typedef struct disco_device_preset {
    double prefill_tok_per_s, decode_tok_per_s;
    float dev_pre_spt_s, dev_dec_spt_s, dev_ttft_c;
    char name[44];
} disco_device_preset;
int32_t disco_device_profile(int32_t index, disco_device_preset* out /*host*/);

/* ---- policy and cost ---------------------------------------------------- */

#define DISCO_MODE_SERVER_CONSTRAINED 0   /* length threshold, Sec. 4.2 Eq. 3 / Alg. 3 */
#define DISCO_MODE_DEVICE_CONSTRAINED 1   /* wait time, Sec. 4.2 Eq. 1 / Alg. 2 */
#define DISCO_MODE_STOCH_SERVER       2   /* baseline Stoch-S, Sec. 5.1: random routing, server budget capped */
#define DISCO_MODE_STOCH_DEVICE       3   /* baseline Stoch-D, Sec. 5.1: random routing, device budget capped */
#define DISCO_MIG_NONE 0
#define DISCO_MIG_LAG  1                  /* hand-off to the device when a server token is overdue */
#define DISCO_MIG_BUFFER 2                /* Sec. 4.3: the constrained endpoint hands decoding over once the token
                                           * buffer hides the hand-off and the saving exceeds the overhead */

/* One policy column (32 bytes).
 * Server-constrained: prompts with l < l_th run on the device alone, the
 *   rest start on both endpoints at time 0 (Alg. 3).
 * Device-constrained: the server starts at 0; the device starts after the
 *   wait w(l) = 0 if l <= l_th; w_mid if l == l_mid; else min(beta * l,
 *   w_tail) -- but only if the server's first token has not arrived by then
 *   (s > w).  beta = +inf gives the step map of Alg. 2, l_mid = -1 the ramp
 *   of Eq. 1, w_tail = +inf a server-only column.
 * In both modes the endpoint with the strictly earlier first token decodes
 * and the other is terminated (Sec. 4.2); a tie goes to the server.
 * Stochastic baselines (Sec. 5.1, Stoch-S / Stoch-D): one endpoint per
 *   request, the constrained one (server for STOCH_SERVER, device for
 *   STOCH_DEVICE) with probability beta = the budget ratio in [0, 1], else
 *   the other; l_mid is the run number.  Request i of a run draws U = ((x >> 9)
 *   + 1/2) 2^-23 from word 0 of Philox4x32-10 with key (run, 0x53544F43) and
 *   counter (i_lo, i_hi, 6, 0) and goes to the constrained endpoint iff
 *   U < beta: columns of one run are nested in beta, runs are independent.
 *   Averaging over runs: disco_average_runs. */
typedef struct disco_policy {
    int32_t mode;
    int32_t l_th;
    int32_t l_mid;
    float w_mid;
    float beta;
    float w_tail;
    int32_t mig_mode;
    int32_t reserved;
} disco_policy;

/* Unified cost (Sec. 4.1, App. E): server money per token plus lambda times
 * device energy per token, prefill and decode priced separately.
 * total = cs_pre*S_pre + cs_dec*S_dec + lambda*(e_pre*D_pre + e_dec*D_dec). */
typedef struct disco_cost_params {
    double cs_pre, cs_dec;   /* $ per server prefill / decode token */
    double e_pre, e_dec;     /* J per device prefill / decode token (linear in FLOPs) */
    double lambda;           /* $ per J */
} disco_cost_params;

/* Policy type (Alg. 1): *mode = DISCO_MODE_DEVICE_CONSTRAINED if the cheaper
 * device token (lambda e_pre or lambda e_dec, in money) costs more than the
 * dearer server token (cs_pre or cs_dec), else DISCO_MODE_SERVER_CONSTRAINED
 * (equality included).  Host only.  Errors: NULL, RANGE (a NaN rate). */
int32_t disco_policy_type(const disco_cost_params* cost /*host*/, int32_t* mode /*host*/);

/* Pacing of the token buffer (Sec. 4.3): tokens leave the buffer no faster
 * than one per `tau` seconds (the user's consumption rate r_c = 1/tau); a
 * lag hand-off fires when a token is more than kappa_lag * tau overdue.
 * cost: host, nullable; the prices behind the buffer hand-off's cost test
 * (columns with DISCO_MIG_BUFFER never hand off without it).
 * reuse_walk: disco_eval_migration (without `delivered`) leaves, in the
 * per-request part of the workspace, what its walk over the token array found
 * for every request (the running maximum of each of its timelines and the
 * lag hand-off, 16 bytes).  A caller who passes the same workspace, untouched
 * by other calls in between except disco_reduce_stats, with the same trace,
 * policy table, tau and kappa_lag to disco_reduce_stats may set reuse_walk = 1:
 * the TBT order statistics then start from those summaries instead of walking
 * the tokens again. */
typedef struct disco_timeline_params {
    float tau;
    float kappa_lag;
    const disco_cost_params* cost;
    int32_t reuse_walk;      /* disco_reduce_stats only, see there; 0: walk the tokens again */
    int32_t reserved;
} disco_timeline_params;

/* ---- per-pair outputs and per-column accumulators ----------------------- */

/* Optional materialised dispatch outputs, device, [P][n_req]; either member
 * may be NULL.  decision: bit0 server started, bit1 device started, bit2
 * device won (1 server only, 6 device only, 3 race won by the server, 7 race
 * won by the device).  ttft: time to first token of the pair. */
typedef struct disco_pair_out {
    uint8_t* decision;
    float* ttft;
} disco_pair_out;

/* Optional materialised timeline outputs, device; members may be NULL.
 * mig_idx [P][n_req]: index of the first token produced by the other
 *   endpoint after a hand-off, -1 if none.  n_src_tok [P][n_req]: tokens
 *   produced by the endpoint that won the first token.  t_last [P][n_req]:
 *   delivery offset of the last token since the first one.  delay_num
 *   [P][n_req]: tokens after a buffer hand-off that arrive after their
 *   pacing slot, r_t > delta_{t-1} + tau (Sec. 5.2, delay_num: the buffer ran
 *   dry and the user waits for them), 0 without hand-off.
 * delivered [n_tok] (column `delivered_col` only; needs tok_off): delivery
 *   offset of every token. */
typedef struct disco_mig_out {
    int32_t* mig_idx;
    int32_t* n_src_tok;
    float* t_last;
    float* delivered;
    int32_t delivered_col;
    int32_t reserved;
    int32_t* delay_num;
} disco_mig_out;

/* Per-column accumulator, device, 128 bytes.  disco_eval_dispatch overwrites
 * the first block, disco_eval_migration the second. */
typedef struct disco_accum {
    /* dispatch: every started endpoint is charged the prompt; the winner is
     * charged the n output tokens (the paper's "w/o Migration" accounting) */
    int64_t s_pre, s_dec, d_pre, d_dec;
    int64_t n_dev_started, n_dev_win;
    double ttft_sum;
    /* timelines: decode tokens per endpoint with hand-offs, extra device
     * re-prefill tokens (prompt + tokens already produced, Sec. 4.3: only
     * token ids are transferred; m_s_repre below is the server's share after
     * buffer hand-offs from the device), hand-off count, number of TBT
     * values, sum of last delivery offsets (= sum of all TBT values) */
    int64_t m_s_dec, m_d_dec, m_d_repre;
    int64_t n_migrated, tbt_count;
    double tlast_sum;
    /* smallest and largest fp32 bit pattern among the column's TTFT values
     * (non-negative floats order like their bit patterns); they bound the key
     * range of the TTFT order-statistic selection */
    uint32_t ttft_min_bits, ttft_max_bits;
    int64_t m_s_repre;        /* timelines: extra server re-prefill tokens */
    int64_t delay_sum;        /* timelines: sum of delay_num over the requests with a buffer hand-off */
} disco_accum;

/* ---- evaluation --------------------------------------------------------- */

/* Dispatch of every (request, column) pair (Sec. 4.2, Alg. 2 and 3):
 * device TTFT d = fma(l, k, c); wait; which endpoints start; winner; TTFT.
 * pol: host or device, P entries.  out: host struct of device arrays, may be NULL.
 * acc: device, P entries, dispatch block overwritten.
 * ws: device workspace of disco_workspace_bytes(n_req, P) bytes.
 * Asynchronous.  n_req == 0 is valid (zero totals).
 * Errors: NULL, SHAPE, RANGE (unknown mode, routing probability outside
 * [0, 1]), WORKSPACE, HIP. */
int32_t disco_eval_dispatch(const disco_trace* trace /*host*/, const disco_policy* pol /*host*/, int32_t P,
                            const disco_pair_out* out /*host, nullable*/, disco_accum* acc /*device*/,
                            void* ws /*device*/, size_t ws_bytes, void* stream);

/* disco_eval_dispatch for callers that cannot allocate device memory or bring
 * a workspace: code under HIP graph capture, tight serving loops, harnesses
 * that forbid allocation.  Same arguments, results and errors as
 * disco_eval_dispatch without `ws`: the partial results (staged policy table,
 * flag words, device-wide totals) live in a fixed area of
 * DISCO_STATIC_SCRATCH_BYTES bytes of device memory inside the library's code
 * object, which every GPU the library runs on holds until the process ends.
 * Limits: P <= DISCO_MAX_COLS (SHAPE beyond it, nothing launched); n_req is
 * not limited by the area.  The call allocates and frees nothing, on the host
 * or the device.  The first call on a device looks up the area's address
 * there (not an allocation; make that call outside a graph capture).  All
 * calls on one GPU share the area: it is put back to its initial state at the
 * start of every call, and calls that overlap in time on one GPU (different
 * streams or threads) race -- serialise them.  Asynchronous. */
#define DISCO_STATIC_SCRATCH_BYTES 133376
int32_t disco_eval_dispatch_static(const disco_trace* trace /*host*/, const disco_policy* pol /*host or device*/, int32_t P,
                                   const disco_pair_out* out /*host, nullable*/, disco_accum* acc /*device*/,
                                   void* stream);

/* Token timelines of every pair (Sec. 4.3).  The source of a pair is the
 * winner of its dispatch (recomputed from `pol`).  Arrival offsets r_t since
 * the first token: server = tok_arr (or t * srv_tbt without a token trace),
 * device = t * g.  Paced delivery delta_0 = 0, delta_t = max(r_t,
 * delta_{t-1} + tau), evaluated as delta_t = fma(t, tau, max_{v<=t}
 * fma(-v, tau, r_v)).  With mig_mode == DISCO_MIG_LAG and a server source:
 * m = first t >= 1 with r_t - (delta_{t-1} + tau) > kappa_lag * tau; the
 * device then produces tokens m.. with r'_t = fma(t - m + 1, g, ((delta_{m-1}
 * + tau) + kappa_lag*tau) + fma(l + m, k, c)).
 * With mig_mode == DISCO_MIG_BUFFER and the column's constrained endpoint as
 * source (server-constrained column: server source, hand-off to the device;
 * device-constrained column: device source, hand-off to the server): the
 * source stops after m = first t < n - 1 with delta_t - r_t >= t_mig(t) (the
 * buffer hides the hand-off) and dc (n - 1 - t) > cp (l + t + 1) in fp64 (the
 * decode saving exceeds the target's prefill overhead; dc = |price difference
 * of a decode token|, cp = target's prefill price, from tl->cost), where
 * t_mig(t) = fma(l + t + 1, k, c) for a device target and the server's TTFT
 * for a server target; the target's tokens arrive at r'_t = fma(t - m, g,
 * r_m + t_mig(m)) (device), fma(t - m, srv_tbt, ...) or (r_m + t_mig(m)) +
 * (tok_arr_t - tok_arr_m) (server without / with a token trace), t > m.
 * Tables with such columns run in a slower, general kernel.
 * acc: device, P entries, timeline block overwritten.  Asynchronous.
 * ws: disco_workspace_bytes(n_req, P) bytes (the per-request part is needed).
 * Errors: NULL, SHAPE, RANGE (tau <= 0, kappa_lag < 0), CSR (delivered
 * requested without tok_off), WORKSPACE, HIP. */
int32_t disco_eval_migration(const disco_trace* trace /*host*/, const disco_timeline_params* tl /*host*/,
                             const disco_policy* pol /*host*/, int32_t P,
                             const disco_mig_out* out /*host, nullable*/, disco_accum* acc /*device*/,
                             void* ws /*device*/, size_t ws_bytes, void* stream);

/* ---- statistics --------------------------------------------------------- */

/* Per-column result (Sec. 5.1 metrics), device or host memory, 256 bytes. */
typedef struct disco_stats {
    double mean_ttft, mean_tbt;
    double server_cost, device_energy, device_cost, total_cost;
    int64_t s_pre, s_dec, d_pre, d_dec;       /* totals used for the cost */
    int64_t n_req, tbt_count, n_migrated, n_dev_started, n_dev_win;
    int64_t ttft_rank[DISCO_MAX_Q];            /* 1-based rank selected for each quantile */
    int64_t tbt_rank[DISCO_MAX_Q];
    float ttft_q[DISCO_MAX_Q];                 /* the order statistic of that rank */
    float tbt_q[DISCO_MAX_Q];
    double mean_delay_num;                     /* delay_sum / n_migrated (NaN without hand-offs or timelines) */
    float delay_q[DISCO_MAX_Q];                /* order statistics of delay_num over the migrated requests (the
                                                * TBT table of Sec. 5.2 reports its mean and P99); counts above
                                                * 8190 are taken as 8191; NaN without hand-offs or timelines */
    int64_t reserved[2];
} disco_stats;

typedef struct disco_quantile { int32_t num, den; } disco_quantile;   /* q = num/den in [0,1] */

/* Reduce the accumulators of the eval calls to per-column statistics and
 * select order statistics.  Quantile q of M values is the nearest-rank order
 * statistic: rank k = ceil(q M) clamped to [1, M], computed in integers;
 * M == 0 gives rank 0 and NaN.  TTFT quantiles are over the n_req pairs of a
 * column; TBT quantiles pool every gap delta_t - delta_{t-1} of every request
 * of the column (sum of n_i - 1 values).  Selection is exact: a most-
 * significant-digit-first radix histogram select over the fp32 bit patterns
 * (times are non-negative, so the patterns order like the values); the pairs
 * are recomputed from the trace for every digit rather than stored.
 * tl == NULL: dispatch statistics only (decode charged to the winner).
 * tl != NULL: acc must also hold disco_eval_migration's block; decode and
 *   re-prefill tokens come from it and TBT statistics are produced.
 * out: device, P entries.  Asynchronous.
 * Errors: NULL, SHAPE (nq outside [0, DISCO_MAX_Q]; TBT quantiles over more
 * than 2^32 - 1 requests), RANGE (den <= 0, num outside [0, den]), WORKSPACE,
 * HIP. */
int32_t disco_reduce_stats(const disco_trace* trace /*host*/, const disco_cost_params* cost /*host*/,
                           const disco_timeline_params* tl /*host, nullable*/,
                           const disco_policy* pol /*host*/, int32_t P,
                           const disco_accum* acc /*device*/, const disco_quantile* q /*host*/, int32_t nq,
                           disco_stats* out /*device*/, void* ws /*device*/, size_t ws_bytes, void* stream);

/* Mean over runs (Sec. 5.1: every experiment is reported as the mean over 10
 * runs; the runs of a stochastic baseline are columns that differ in l_mid).
 * in: device, groups * runs records, the runs of group g at g*runs ..
 * g*runs + runs - 1; out: device, groups records (must not overlap in).
 * Floating-point fields: arithmetic mean in fp64, summed in run order (order
 * statistics: the fp64 mean of the fp32 values, rounded to fp32; NaN
 * propagates); integer totals and counts: summed over the runs; ranks: those
 * of the first run.  Asynchronous.  Errors: NULL, SHAPE (groups < 0, runs < 1),
 * HIP. */
int32_t disco_average_runs(const disco_stats* in /*device*/, int32_t groups, int32_t runs,
                           disco_stats* out /*device*/, void* stream);

/* ---- closed-form policy solves ------------------------------------------ */

/* One column to solve.  b = b_num / b_den in [0, 1] is the budget ratio: the
 * constrained endpoint's share of the prompt tokens (Sec. 4.2); alpha = a_num /
 * a_den in (0, 1) the tail ratio of Alg. 2 (ignored for Alg. 3).  Denominators
 * in [1, 32768], so that every budget comparison is exact in 128-bit integers. */
typedef struct disco_solve_spec {
    int32_t mode;            /* DISCO_MODE_SERVER_CONSTRAINED: Alg. 3; DISCO_MODE_DEVICE_CONSTRAINED: Alg. 2 */
    int32_t b_num, b_den;
    int32_t a_num, a_den;
    int32_t mig_mode;        /* copied into the policy record */
    int32_t reserved[2];
} disco_solve_spec;

/* What the solve used, per column (device). */
typedef struct disco_solve_out {
    int64_t rank_tail;        /* Alg. 2: rank of the server TTFT taken as w_tail (0: wait 0) */
    int64_t rank_mid;         /* Alg. 2: rank of the partial wait (0: no partial length) */
    int64_t zero_wait_tokens; /* Alg. 2: prompt tokens of the lengths that start the device at once;
                               * Alg. 3: prompt tokens of the device-only prompts */
    int64_t total_tokens;
    int32_t status;           /* 1: the trace has prompts of 32772 tokens or more, which the length table
                               * does not hold: the record is not the solve's answer */
    int32_t reserved[3];
} disco_solve_out;

/* Policy columns for budget levels as the paper's dispatch controller solves
 * them (Sec. 4.2), with the trace's own distributions: p(l) = requests per
 * prompt length, F = empirical distribution of the server TTFT, taken as
 * independent of each other; F^-1(q) is the order statistic of rank
 * ceil(q n_req), rank 0 gives 0.
 * Alg. 3 / Eq. 3: l_th = the smallest L such that the prompts of length >= L
 *   hold at most b of the prompt tokens (they race; shorter ones run on the
 *   device alone).
 * Alg. 2: w_tail = F^-1(1 - min(alpha, b)); if b <= alpha every length waits
 *   w_tail.  Otherwise (b - alpha) x total tokens are spent in ascending
 *   order of length: a length costs (1 - alpha) x its tokens and gets wait 0
 *   (l_th = the last such length); the first length that is not affordable,
 *   l_mid, waits w_mid = F^-1((1 - alpha) - left / its tokens) -- the extra
 *   device prefill at that wait is what is left; the printed equation for this
 *   wait has the opposite monotonic direction and is read this way.  The
 *   record has beta = +inf (step map).
 * pol_out: device, n records; out: device, n records, nullable.  Prompt
 * lengths must be positive and below 32772 (out.status otherwise), server
 * TTFTs non-negative.  Asynchronous.  Errors: NULL, SHAPE (n outside [1,
 * DISCO_MAX_COLS]), RANGE (unknown mode, ratios outside their ranges,
 * denominators outside [1, 32768]), WORKSPACE, HIP. */
int32_t disco_solve_policy(const disco_trace* trace /*host*/, const disco_solve_spec* spec /*host*/, int32_t n,
                           disco_policy* pol_out /*device*/, disco_solve_out* out /*device, nullable*/,
                           void* ws /*device*/, size_t ws_bytes, void* stream);

/* ---- budget search ------------------------------------------------------ */

#define DISCO_PARAM_L_TH    0   /* integer bisection on disco_policy.l_th */
#define DISCO_PARAM_W_TAIL  1   /* fp32 bisection on disco_policy.w_tail */
#define DISCO_PARAM_BETA    2   /* fp32 bisection on disco_policy.beta: the ramp slope of Eq. 1, root of Eq. 2 on the trace */

#define DISCO_ACC_TOTAL_COST          0
#define DISCO_ACC_SERVER_COST         1
#define DISCO_ACC_DEVICE_COST         2   /* lambda * device energy */
#define DISCO_ACC_SERVER_PREFILL_TOK  3   /* input tokens the server processes (budget of Eq. 3) */
#define DISCO_ACC_DEVICE_PREFILL_TOK  4   /* input tokens the device processes (budget of Sec. 4.2) */

/* One search: bisect one parameter of `templ` so that an accumulator that
 * does not increase with the parameter meets `target` (the budget of Sec. 4.2
 * is an allowance for the constrained endpoint; Eq. 3 and Alg. 2 ask for the
 * threshold / wait that meets it).  The accumulator is computed from exact
 * int64 token totals of a dispatch pass (decode charged to the winner).
 * W_TAIL, BETA: mid = 0.5f * (lo + hi) in fp32; A(mid) > target ? lo = mid : hi = mid;
 *   after n_steps the answer is hi.  (BETA: the slope of the ramp min(beta l, w_tail) of Eq. 1 for the prompts
 *   above l_th; with which_acc = DEVICE_PREFILL_TOK and target = what is left of the budget this is Eq. 2, its
 *   left-hand side taken on the trace.)
 * L_TH: mid = lo + (hi - lo) / 2; while lo < hi: A(mid) > target ? lo = mid + 1
 *   : hi = mid; later steps re-evaluate at the answer hi.
 * The caller guarantees A(hi) <= target at entry (e.g. hi = longest prompt + 1
 * for L_TH). */
typedef struct disco_search_spec {
    int32_t which_param;
    int32_t which_acc;
    int32_t n_steps;      /* 1 .. DISCO_MAX_STEPS */
    int32_t reserved;
    double lo, hi;
    double target;
} disco_search_spec;

/* Result of one search, device memory. */
typedef struct disco_search_out {
    double param;                         /* the answer (hi) */
    double acc_at_param;                  /* accumulator re-evaluated at the answer */
    double lo, hi;                        /* final bracket */
    double hist_param[DISCO_MAX_STEPS];   /* midpoint tried at each step */
    double hist_acc[DISCO_MAX_STEPS];     /* accumulator at that midpoint */
    disco_accum at_param;                 /* dispatch totals at the answer */
} disco_search_out;

/* Run n_search independent searches over the same trace.  In general every
 * step is one fused dispatch-and-reduce pass that evaluates all searches'
 * midpoints; the brackets are updated on the device, so there is no host
 * round trip between steps.  When every search is a length threshold of a
 * server-constrained template (Alg. 3) against a prompt-token accumulator,
 * with 0 <= lo and hi <= 32770, the accumulator is tabulated for every
 * threshold in one pass (Alg. 3's running totals over the sorted lengths)
 * and the steps read the table; results and recorded history are the same.
 * All searches must have the same n_steps.
 * templ, spec: host, n_search entries.  out: device, n_search entries.
 * pol_out: device, n_search entries (nullable): the template with the found
 * parameter, ready to be copied into a policy table.
 * acc_out: device, n_search entries (nullable): the dispatch block of the
 * accumulators at the answer, exactly what disco_eval_dispatch would leave
 * for pol_out (the search's last pass is that evaluation), so a caller that
 * goes on to disco_reduce_stats need not evaluate again.
 * Asynchronous.  Errors: NULL, SHAPE (n_search outside [1, DISCO_MAX_COLS],
 * n_steps out of range or unequal), RANGE (unknown selector, lo > hi, a
 * stochastic baseline as template),
 * WORKSPACE, HIP. */
int32_t disco_budget_search(const disco_trace* trace /*host*/, const disco_cost_params* cost /*host*/,
                            const disco_policy* templ /*host*/, const disco_search_spec* spec /*host*/,
                            int32_t n_search, disco_search_out* out /*device*/,
                            disco_policy* pol_out /*device, nullable*/, disco_accum* acc_out /*device, nullable*/,
                            void* ws /*device*/, size_t ws_bytes, void* stream);

/* ---- helpers ------------------------------------------------------------ */

/* Bytes of device workspace for n_req requests and P columns (or searches):
 * about 47 MB plus 61 bytes per request.  The per-request part (one byte that
 * the TTFT selection and the token walk use between their passes, 16 bytes of
 * what the token walk found, 32 bytes of the same for buffer hand-offs, 12 bytes
 * of the TBT selection) is needed by
 * disco_eval_migration and by
 * disco_reduce_stats with timelines; every other call accepts a workspace of
 * disco_workspace_bytes(0, P) bytes.  The workspace holds partial results
 * only; its contents need not be initialised or preserved between calls
 * (except for reuse_walk, see disco_timeline_params), and calls that share
 * one workspace must not overlap in time.  It must be ordinary (coarse-grained) device memory,
 * 256-byte aligned: the kernels use hardware floating-point atomics on it. */
size_t disco_workspace_bytes(int64_t n_req, int32_t P);

/* Measurement aid (no part of the method): one read-and-reduce pass over
 * `bytes` bytes of device memory (16-byte aligned, a multiple of 16), i.e. what
 * the GPU sustains on a plain streaming read; the benchmark quotes it beside
 * the HBM fractions of the token walk.  out64: device, 64 words the kernel may
 * store to (it keeps the reads from being elided).  Asynchronous.
 * Errors: NULL, SHAPE, HIP. */
int32_t disco_read_probe(const void* src /*device*/, int64_t bytes, void* out64 /*device*/, void* stream);

/* Measurement aid: runs the token-walk part of disco_eval_migration (which
 * requests to walk, the streaming walk over the token array, the exact
 * re-walk of the few requests it leaves) reps + 1 times and reports the mean
 * and the minimum duration, in milliseconds, of the streaming kernel alone
 * over the last reps runs, taken with HIP events on `stream` around that
 * kernel's launch.  SYNCHRONISES.  mean_ms, min_ms: host.  Needs a trace with
 * a token array.  Errors: as disco_eval_migration; SHAPE (reps outside
 * [1, 1000]), CSR (no token array or no request). */
int32_t disco_time_token_walk(const disco_trace* trace /*host*/, const disco_timeline_params* tl /*host*/,
                              const disco_policy* pol /*host or device*/, int32_t P, void* ws /*device*/, size_t ws_bytes,
                              int32_t reps, double* mean_ms /*host*/, double* min_ms /*host*/, void* stream);

/* Testing aid: from now on the grids of the dispatch pass and of the token
 * walk are divided by d (1 = the normal geometry) before launch, process-wide.
 * Integer results must not depend on it.  Errors: RANGE (d outside [1, 1024]). */
int32_t disco_set_grid_divisor(int32_t d);

const char* disco_strerror(int32_t code);
const char* disco_last_hip_error(void);   /* text of the last HIP failure seen by this thread */
int32_t disco_version(void);

#ifdef __cplusplus
}
#endif
#endif /* DISCO_H */
