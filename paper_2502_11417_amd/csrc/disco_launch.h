// Host-side launch interface between the translation units of libdisco.
#pragma once
#include "disco_state.h"

// dc = price difference of a decode token (source minus target), cp = target's prefill price; _srv: server
// source handing off to the device, _dev: device source handing off to the server.
struct BufCostArgs { double dc_srv, cp_srv, dc_dev, cp_dev; };

struct TimelineArgs {
    float tau, kt;            // pacing interval, kappa_lag * tau
    int P, nq, pass;          // -1: statistics pass, >= 0: TBT histogram pass
    int32_t* mig_idx; int32_t* n_src_tok; float* t_last; float* delivered; int delivered_col;
    MigPartial* part; unsigned* ticket; disco_accum* acc;
    SelState* S; unsigned* ghist;
    unsigned* ppcnt;          // pure-pacing timelines per class and length (histogram passes)
    int32_t* delay_num;       // materialised delayed-token counts (buffer hand-off), nullable
    BufCostArgs bc;           // prices of the buffer hand-off's cost test
    const unsigned* buffer_flag;   // device: 1 if the staged table has a buffer hand-off column
    unsigned* dhist;               // histogram passes: migrated requests by number of delayed tokens, per column
    unsigned char* wflags;         // one byte per request: the walks it needs (written by the statistics pass)
    void* summary;                 // TlSummary per request: what the token walk found (16 bytes each)
    unsigned* counter;             // batch counters of the token walk, one per queue (zeroed by the flags kernel)
    u64* desc;                     // per request: LDS rows of its timelines with tokens to walk, one byte per kind (histogram passes)
    void* bufsum;                  // BufSummary per request: what the walk of its buffer hand-off timelines found
    unsigned* list;                // the requests that have such a timeline, one word each (histogram passes)
};

// How the last workgroup of a dispatch pass hands on the column totals.
struct DispFin {
    int kind;                     // 0: write disco_accum, 1: advance a budget search
    int need;                     // totals wanted: 0 prefill tokens, 1 + decode split, 2 + TTFT sum and range
    disco_accum* acc;
    disco_cost_params cost;
    SearchState* st;
    disco_search_out* sout;
    disco_policy* pol_out;
    disco_policy* pol_rw;         // the table the next pass reads
    // Bisection passes of a search evaluate a whole subtree of the bisection at once: search j owns the
    // 2^depth - 1 columns j * (2^depth - 1) ..., one per node of the next `depth` levels (heap order), so one pass
    // takes `depth` bisection steps; depth 0: the columns are the searches themselves (final evaluation).
    int n_search, depth;
    int last;                     // the last bisection pass: leave the answers' policies in pol_rw[0 .. n_search)
    const disco_policy* templ;    // the searches' template records
};

// Levels of the bisection tree one pass can evaluate for n searches (64 columns per pass).
inline int disco_search_depth(int n) { return n <= 9 ? 3 : (n <= 21 ? 2 : 1); }

void disco_launch_dispatch_acc(const TraceView& v, const disco_policy* pol, int P, u64* part, const DispFin& fin,
                               hipStream_t stream);
// Threshold search of server-constrained columns from a table of prompt-token sums by length.
void disco_launch_search_table(const TraceView& v, int n_search, int nbins, unsigned* scratch, size_t scratch_bytes,
                               u64* table, u64* other, SearchState* st, disco_policy* pol, disco_search_out* sout,
                               hipStream_t stream);
int disco_search_table_max_bins(void);
void disco_launch_len_table(const TraceView& v, int nbins, unsigned* scratch, size_t scratch_bytes, u64* table, u64* other,
                            hipStream_t stream);
// Pairs with the buffer hand-off in class mode: their per-request summaries (a.bufsum), from the summaries of the
// streaming walk (a.summary) and the tokens; returns at once when the staged table has no such column.
// `totals` nullable: summaries only.
void disco_launch_tl_stats_buf(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a,
                               MigPartial* totals, hipStream_t stream);
// Recorded traces: timestamps to relative arrays; log-normal fit (`scratch`: disco_fit_scratch_bytes() bytes).
void disco_launch_ingest(i64 n_req, const double* t_send, const double* t_token, const i64* off, float* srv_ttft,
                         int32_t* output_len, float* tok_arr, hipStream_t stream);
size_t disco_fit_scratch_bytes(void);
void disco_launch_fit(const void* x, int kind, i64 n, disco_lognormal_fit* fit, void* scratch, hipStream_t stream);
// Closed-form policy solves (Alg. 2, Alg. 3): length table, per-column plan, multi-rank selection over the server
// TTFTs, policy records.  `state` needs disco_solve_state_bytes() bytes.
size_t disco_solve_state_bytes(void);
void disco_launch_solve(const TraceView& v, const disco_solve_spec* spec, int n, void* state, u64* table, u64* other,
                        unsigned* scratch, size_t scratch_bytes, disco_policy* pol_out, disco_solve_out* out,
                        hipStream_t stream);
// One TTFT radix pass: histograms per workgroup slice (class kernel or pair kernel, decided on the device),
// row sums, digit selection.
// `ubytes`: n_req bytes of scratch (nullable) where the first pass leaves, per request, the number of thresholds
// not above its prompt length for the later passes.
void disco_launch_ttft_pass(const TraceView& v, const disco_policy* pol, int P, int nq, int pass, SelState* S,
                            unsigned* slices, unsigned* rowsum, unsigned char* ubytes, hipStream_t stream);
void disco_launch_dispatch_mat(const TraceView& v, const disco_policy* pol, int P, uint8_t* decision, float* ttft,
                               hipStream_t stream);
// Token timelines.  Statistics pass (a.pass = -1): streaming kernel, or the general kernel when the
// per-token deliveries of a column are wanted.  TBT selection: classification, assignment and the "longer than"
// counts of the analytic timelines once; then per regular pass (a.pass < DISCO_TBT_REGULAR_PASS) the walk of the
// streaming kinds (disco_launch_tl_hist_fast) followed by disco_launch_tbt_pass (the other histogram work of the
// pass, the digits, the plan of the next pass); a spare pass is disco_launch_tbt_pass alone, one launch that
// normally returns at once.
void disco_launch_tl_stats_fast(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a,
                                MigPartial* totals, hipStream_t stream);
// The token walk alone (flags, then one 16-byte summary per request), for a statistics call that was not handed
// the summaries of the evaluation.
void disco_launch_tl_walk(const TraceView& v, i64 n_tok, const disco_policy* pol, int P, float tau, float kt,
                          unsigned char* wflags, void* summary, unsigned* counter, hipStream_t stream,
                          hipEvent_t before = nullptr, hipEvent_t after = nullptr);
void disco_launch_timeline_general(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a,
                                   hipStream_t stream);
void disco_launch_tl_classify(const TraceView& v, const disco_policy* pol, int P, int nq, float tau, const void* summary,
                              const void* bufsum, SelState* S, unsigned* ppcnt, unsigned* ghist, unsigned* dhist,
                              unsigned* ticket, hipStream_t stream);
void disco_launch_tl_hist_fast(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a,
                               hipStream_t stream);
void disco_launch_tl_assign(const TraceView& v, const disco_policy* pol, int P, const void* summary, SelState* S,
                            const void* bufsum, u64* desc, unsigned* list, unsigned* slices, size_t slices_bytes,
                            unsigned* ppcnt, unsigned* dhist, hipStream_t stream);
void disco_launch_pp_suffix(SelState* S, unsigned* ppcnt, hipStream_t stream);
void disco_launch_tbt_pass(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a, hipStream_t stream);
