// Host-side helpers of libdisco: HIP error capture and workspace layout.
#pragma once
#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>
#include "disco.h"

void disco_set_hip_error(hipError_t e, const char* what);

#define DISCO_HIP(expr)                                   \
    do {                                                  \
        hipError_t e_ = (expr);                           \
        if (e_ != hipSuccess) {                           \
            disco_set_hip_error(e_, #expr);               \
            return DISCO_ERR_HIP;                         \
        }                                                 \
    } while (0)

// Testing aid: every grid of the dispatch pass and of the token walk is divided by this (>= 1) before launch, so
// that a test can run the same input under two launch geometries and compare the results bit for bit.
int disco_grid_divisor();

// Launch geometry shared by the streaming kernels.
enum {
    DISCO_BLOCK = 256,           // threads per workgroup (4 waves)
    DISCO_MAX_BLOCKS = 2048,     // upper bound of workgroups per launch (8 per CU on 256 CUs)
    DISCO_MAX_SLOTS = 128,       // (columns x quantiles) selected together
    DISCO_FLAG_BUFFER = 40,      // word of the ticket region: 1 if the staged policy table has a buffer hand-off column
};

// Workspace carve-up.  Every region is 256-byte aligned.
struct WsLayout {
    size_t pol;        // disco_policy[64]
    size_t ticket;     // unsigned[64] counters (zeroed by the library before use)
    size_t search;     // SearchState[64]
    size_t sel;        // select state (globals + slots)
    size_t ghist;      // unsigned[DISCO_GHIST_WORDS] device-wide histogram bins
    size_t part;       // device-wide totals (dispatch, then timeline), per-workgroup partials of the general timeline kernel
    size_t ppcnt;      // unsigned[DISCO_MAX_CLS][DISCO_PP_NMAX + 1]: pure-pacing timelines per class and length
    size_t dhist;      // unsigned[DISCO_MAX_COLS][DISCO_DELAY_BINS]: migrated requests by number of delayed tokens
    size_t templ;      // disco_policy[64]: templates of a budget search (its candidate columns are in `pol`)
    size_t wcount;     // unsigned[1024]: batch counters of the token walk, one per queue, 128 bytes apart
    size_t slices;     // per-workgroup histogram slices (TTFT passes, prompt-length table): 32 MB
    size_t total;
};
WsLayout disco_ws_layout(int32_t P);
// Behind the fixed regions: one byte per request (TTFT selection: thresholds not above the prompt length; token
// walk: which timelines to walk), then 16 bytes per request (what the token walk found), then 32 bytes per request (what the walk of its
// buffer hand-off timelines found), then 12 bytes per request (TBT selection: which of its timelines have tokens to
// walk and into which histogram rows; the list of such requests).
inline size_t disco_ws_bytes_region(int64_t n_req) { return n_req > 0 ? (((size_t)n_req + 255) & ~(size_t)255) : 0; }
inline size_t disco_ws_summary_offset(const WsLayout& L, int64_t n_req) { return L.total + disco_ws_bytes_region(n_req); }
inline size_t disco_ws_bufsum_offset(const WsLayout& L, int64_t n_req)
{
    return disco_ws_summary_offset(L, n_req) + (n_req > 0 ? (size_t)n_req * 16 : 0);
}
inline size_t disco_ws_desc_offset(const WsLayout& L, int64_t n_req)
{
    return disco_ws_bufsum_offset(L, n_req) + (n_req > 0 ? (size_t)n_req * 32 : 0);
}
inline size_t disco_ws_full_bytes(const WsLayout& L, int64_t n_req)
{
    return disco_ws_desc_offset(L, n_req) + (n_req > 0 ? (size_t)n_req * 12 : 0);     // descriptors (8), then the walk list (4)
}
