// Opt-in validation of a trace before it is evaluated (recorded traces enter through disco_ingest_trace; the
// evaluation kernels trust the arrays they are given: a token offset that does not match the output length
// makes them read outside the token array).  One pass over the requests, then -- if the offsets are sound, so
// that the pass cannot leave the token array -- one pass over the tokens.  Findings are OR-ed into one word.
#include <math.h>

#include "disco_common.h"
#include "disco_device.h"

namespace {

enum { BAD_CSR = 1, BAD_RANGE = 2 };

constexpr int VD_BLOCK = 256;
constexpr int VD_WAVES = VD_BLOCK / 64;

__device__ __forceinline__ bool bad_time(float x) { return !(x >= 0.0f) || x == INFINITY; }      // negative, NaN or infinite

// Requests: lengths, times and rates in range; offsets start at 0, advance by the output length and, with a token
// array, end at n_tok.
__global__ __launch_bounds__(VD_BLOCK) void k_validate_requests(TraceView tr, i64 n_tok, const i64* __restrict__ tok_off,
                                                                 unsigned* __restrict__ flag)
{
    unsigned bad = 0u;
    for (i64 i = (i64)blockIdx.x * blockDim.x + threadIdx.x; i < tr.n_req; i += (i64)gridDim.x * blockDim.x) {
        const int l = tr.l[i], n = tr.n[i];
        if (l < 0 || n < 1) bad |= BAD_RANGE;
        if (bad_time(tr.s[i])) bad |= BAD_RANGE;
        if (tr.tbt && bad_time(tr.tbt[i])) bad |= BAD_RANGE;
        if (tr.k && bad_time(tr.k[i])) bad |= BAD_RANGE;
        if (tr.g && bad_time(tr.g[i])) bad |= BAD_RANGE;
        if (tok_off) {
            const i64 a = tok_off[i], b = tok_off[i + 1];
            if (a < 0 || b < a || b - a != (i64)n) bad |= BAD_CSR;
            if (i == 0 && a != 0) bad |= BAD_CSR;
            if (tr.arr && (b > n_tok || (i == tr.n_req - 1 && b != n_tok))) bad |= BAD_CSR;      // (n_tok counts a token array)
        }
    }
    if (__ballot(bad != 0u) != 0ull) {
        const unsigned all = (__ballot((bad & BAD_CSR) != 0u) ? (unsigned)BAD_CSR : 0u) |
                             (__ballot((bad & BAD_RANGE) != 0u) ? (unsigned)BAD_RANGE : 0u);
        if ((threadIdx.x & 63) == 0) atomicOr(flag, all);
    }
}

// Tokens (offsets already found sound): arrival offsets start at 0, never decrease inside a request, are finite.
// One wave per request, lanes stride its tokens.
__global__ __launch_bounds__(VD_BLOCK) void k_validate_tokens(i64 n_req, const i64* __restrict__ tok_off, const float* __restrict__ arr,
                                                               unsigned* __restrict__ flag)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    bool bad = false;
    for (i64 i = (i64)blockIdx.x * VD_WAVES + wave; i < n_req; i += (i64)gridDim.x * VD_WAVES) {
        const i64 a = tok_off[i], b = tok_off[i + 1];
        for (i64 j = a + lane; j < b; j += 64) {
            const float x = arr[j];
            if (bad_time(x)) bad = true;
            if (j == a ? x != 0.0f : arr[j - 1] > x) bad = true;
        }
    }
    if (__ballot(bad) != 0ull && lane == 0) atomicOr(flag, (unsigned)BAD_RANGE);
}

}  // namespace

extern "C" int32_t disco_validate_trace(const disco_trace* t, int32_t check_tokens, void* ws_, size_t ws_bytes, void* stream_)
{
    if (!t) return DISCO_ERR_NULL;
    if (t->n_req < 0 || t->n_tok < 0) return DISCO_ERR_SHAPE;
    if (t->n_req > 0 && (!t->prompt_len || !t->output_len || !t->srv_ttft)) return DISCO_ERR_NULL;
    if ((t->tok_arr != nullptr) && !t->tok_off) return DISCO_ERR_CSR;
    if (!ws_ || ws_bytes < 256 || ((uintptr_t)ws_ & 255u) != 0) return DISCO_ERR_WORKSPACE;
    if (!(t->dev_ttft_c >= 0.0f) || (!t->dev_pre_spt && !(t->dev_pre_spt_s >= 0.0f)) || (!t->dev_dec_spt && !(t->dev_dec_spt_s >= 0.0f)))
        return DISCO_ERR_RANGE;
    if (t->n_req == 0) return t->n_tok == 0 || !t->tok_off ? DISCO_OK : DISCO_ERR_CSR;
    hipStream_t stream = (hipStream_t)stream_;
    unsigned* flag = (unsigned*)ws_;
    TraceView v;
    v.n_req = t->n_req;
    v.l = t->prompt_len; v.n = t->output_len; v.s = t->srv_ttft; v.tbt = t->srv_tbt;
    v.k = t->dev_pre_spt; v.g = t->dev_dec_spt; v.off = t->tok_off; v.arr = t->tok_arr;
    v.k_s = t->dev_pre_spt_s; v.g_s = t->dev_dec_spt_s; v.c = t->dev_ttft_c;
    unsigned found = 0u;
    DISCO_HIP(hipMemcpyAsync(flag, &found, sizeof(found), hipMemcpyHostToDevice, stream));
    i64 b = (t->n_req + VD_BLOCK - 1) / VD_BLOCK;
    if (b > 4096) b = 4096;
    hipLaunchKernelGGL(k_validate_requests, dim3((unsigned)b), dim3(VD_BLOCK), 0, stream, v, t->n_tok, t->tok_off, flag);
    DISCO_HIP(hipGetLastError());
    DISCO_HIP(hipMemcpyAsync(&found, flag, sizeof(found), hipMemcpyDeviceToHost, stream));
    DISCO_HIP(hipStreamSynchronize(stream));
    if (found & BAD_CSR) return DISCO_ERR_CSR;
    if (check_tokens && t->tok_arr) {                        // the offsets are sound: the pass stays inside the token array
        i64 wb = (t->n_req + VD_WAVES - 1) / VD_WAVES;
        if (wb > 8192) wb = 8192;
        hipLaunchKernelGGL(k_validate_tokens, dim3((unsigned)wb), dim3(VD_BLOCK), 0, stream, t->n_req, t->tok_off, t->tok_arr, flag);
        DISCO_HIP(hipGetLastError());
        unsigned found2 = 0u;
        DISCO_HIP(hipMemcpyAsync(&found2, flag, sizeof(found2), hipMemcpyDeviceToHost, stream));
        DISCO_HIP(hipStreamSynchronize(stream));
        found |= found2;
    }
    return (found & BAD_RANGE) ? DISCO_ERR_RANGE : DISCO_OK;
}
