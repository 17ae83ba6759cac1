// Recorded traces (Sec. 5.1: the evaluation is driven by traces of production
// services and on-device profiles) and the log-normal fit of the scalability
// study (Sec. 5.3: prompt length and server TTFT laws fitted by the mean and
// standard deviation of the logarithm).
//
//   k_ingest        wall-clock timestamps -> server TTFT, output length and
//                   token arrival offsets relative to the request's first token:
//                   one wave per request, lanes stride its tokens; a difference
//                   is taken in fp64 and rounded once to fp32.  Streams 12 B per
//                   token (8 read, 4 written).
//   k_fit_sum / k_fit_final   mean of ln x, then mean squared deviation, each a
//                   grid-stride pass with per-workgroup partial sums folded in a
//                   fixed order by one workgroup (the result does not depend on
//                   the order in which workgroups finish).
#include <math.h>
#include <string.h>

#include "disco_launch.h"
#include "disco_device.h"

namespace {

constexpr int IG_BLOCK = 256;
constexpr int IG_WAVES = IG_BLOCK / 64;
constexpr int FIT_BLOCK = 256;
constexpr int FIT_MAX_BLOCKS = 1024;

__global__ __launch_bounds__(IG_BLOCK) void k_ingest(i64 n_req, const double* __restrict__ t_send,
                                                     const double* __restrict__ t_token, const i64* __restrict__ off,
                                                     float* __restrict__ srv_ttft, int32_t* __restrict__ output_len,
                                                     float* __restrict__ tok_arr)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    for (i64 i = (i64)blockIdx.x * IG_WAVES + wave; i < n_req; i += (i64)gridDim.x * IG_WAVES) {
        const i64 a = off[i], b = off[i + 1];
        if (b <= a) {                                   // a request without tokens has no first token
            if (lane == 0) { output_len[i] = 0; srv_ttft[i] = NAN; }
            continue;
        }
        const double first = t_token[a];
        if (lane == 0) {
            output_len[i] = (int32_t)(b - a);
            srv_ttft[i] = (float)(first - t_send[i]);
        }
        // two timestamps per lane and step (16-byte loads, 8-byte stores) from the first even token on
        const i64 a2 = (a + 1) & ~(i64)1;
        if (lane == 0 && a2 > a) tok_arr[a] = 0.0f;
        const bool pair_ok = ((((uintptr_t)t_token) & 15u) == 0) && ((((uintptr_t)tok_arr) & 7u) == 0);
        if (pair_ok) {
            i64 j = a2 + 2 * lane;
            for (; j + 1 < b; j += 128) {
                const double2 v = *reinterpret_cast<const double2*>(t_token + j);
                float2 o;
                o.x = (float)(v.x - first); o.y = (float)(v.y - first);
                *reinterpret_cast<float2*>(tok_arr + j) = o;
            }
            if (j < b) tok_arr[j] = (float)(t_token[j] - first);
        } else {
            for (i64 j = a2 + lane; j < b; j += 64) tok_arr[j] = (float)(t_token[j] - first);
        }
    }
}

struct FitPartial { double sum; u64 used; };

__device__ __forceinline__ double value_of(const void* x, int kind, i64 i)
{
    return kind == 0 ? (double)((const int32_t*)x)[i] : (double)((const float*)x)[i];
}

// pass 0: sum of ln x; pass 1: sum of (ln x - mu)^2 with mu from pass 0.
__global__ __launch_bounds__(FIT_BLOCK) void k_fit_sum(const void* __restrict__ x, int kind, i64 n, int pass,
                                                       const disco_lognormal_fit* fit, FitPartial* part)
{
    __shared__ double ssum[FIT_BLOCK / 64];
    __shared__ u64 sused[FIT_BLOCK / 64];
    const double mu = pass ? fit->mu : 0.0;
    double sum = 0.0;
    u64 used = 0;
    for (i64 i = (i64)blockIdx.x * FIT_BLOCK + threadIdx.x; i < n; i += (i64)gridDim.x * FIT_BLOCK) {
        const double v = value_of(x, kind, i);
        if (v > 0.0) {                                  // NaN and non-positive values have no logarithm
            const double lv = log(v);
            const double dv = lv - mu;
            sum += pass ? dv * dv : lv;
            used += 1;
        }
    }
    sum = wave_sum_f64(sum);
    used = wave_sum_u64(used);
    if ((threadIdx.x & 63) == 0) { ssum[threadIdx.x >> 6] = sum; sused[threadIdx.x >> 6] = used; }
    __syncthreads();
    if (threadIdx.x == 0) {
        FitPartial p{0.0, 0};
        for (int w = 0; w < FIT_BLOCK / 64; ++w) { p.sum += ssum[w]; p.used += sused[w]; }
        part[blockIdx.x] = p;
    }
}

__global__ __launch_bounds__(64) void k_fit_final(int nblocks, i64 n, int pass, const FitPartial* part, disco_lognormal_fit* fit)
{
    double sum = 0.0;
    u64 used = 0;
    for (int b = threadIdx.x; b < nblocks; b += 64) { sum += part[b].sum; used += part[b].used; }
    sum = wave_sum_f64(sum);
    used = wave_sum_u64(used);
    if (threadIdx.x != 0) return;
    if (pass == 0) {
        fit->mu = used ? sum / (double)used : NAN;
        fit->sigma = NAN;
        fit->n_used = (i64)used;
        fit->n_skipped = n - (i64)used;
    } else {
        fit->sigma = used ? sqrt(sum / (double)used) : NAN;
    }
}

// On-device configurations of Sec. 5.1: prefill / decode speed in tokens per second.
const double kProfiles[3][2] = {{31.32, 13.93}, {51.80, 20.14}, {79.90, 21.47}};
const char* const kProfileNames[3] = {"Pixel 7 Pro / Bloom 1.1B", "Pixel 7 Pro / Bloom 560M", "Xiaomi 14 / Qwen 1.5 0.5B"};

}  // namespace

void disco_launch_ingest(i64 n_req, const double* t_send, const double* t_token, const i64* off, float* srv_ttft,
                         int32_t* output_len, float* tok_arr, hipStream_t stream)
{
    i64 b = (n_req + IG_WAVES - 1) / IG_WAVES;
    if (b < 1) b = 1;
    if (b > 8192) b = 8192;
    hipLaunchKernelGGL(k_ingest, dim3((unsigned)b), dim3(IG_BLOCK), 0, stream, n_req, t_send, t_token, off, srv_ttft,
                       output_len, tok_arr);
}

size_t disco_fit_scratch_bytes(void) { return sizeof(FitPartial) * FIT_MAX_BLOCKS; }

void disco_launch_fit(const void* x, int kind, i64 n, disco_lognormal_fit* fit, void* scratch, hipStream_t stream)
{
    i64 b = (n + FIT_BLOCK - 1) / FIT_BLOCK;
    if (b < 1) b = 1;
    if (b > FIT_MAX_BLOCKS) b = FIT_MAX_BLOCKS;
    FitPartial* part = (FitPartial*)scratch;
    for (int pass = 0; pass < 2; ++pass) {
        hipLaunchKernelGGL(k_fit_sum, dim3((unsigned)b), dim3(FIT_BLOCK), 0, stream, x, kind, n, pass, fit, part);
        hipLaunchKernelGGL(k_fit_final, dim3(1), dim3(64), 0, stream, (int)b, n, pass, part, fit);
    }
}

extern "C" int32_t disco_device_profile(int32_t index, disco_device_preset* out)
{
    if (!out) return DISCO_ERR_NULL;
    if (index < 0 || index >= 3) return DISCO_ERR_RANGE;
    memset(out, 0, sizeof(*out));
    out->prefill_tok_per_s = kProfiles[index][0];
    out->decode_tok_per_s = kProfiles[index][1];
    out->dev_pre_spt_s = (float)(1.0 / kProfiles[index][0]);
    out->dev_dec_spt_s = (float)(1.0 / kProfiles[index][1]);
    out->dev_ttft_c = 0.0f;
    strncpy(out->name, kProfileNames[index], sizeof(out->name) - 1);
    return DISCO_OK;
}
