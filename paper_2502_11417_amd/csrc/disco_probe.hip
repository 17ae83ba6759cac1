// Streaming-read probe: what this GPU sustains on a plain read-and-reduce pass, to be quoted beside the
// HBM fractions of the token walk ("fraction of achievable" next to "fraction of peak").
#include "disco_common.h"
#include "disco_device.h"

namespace {

constexpr int RP_BLOCK = 256;
constexpr int RP_UNROLL = 8;                 // 16-byte loads in flight per lane
typedef unsigned Vec4 __attribute__((ext_vector_type(4)));

// Every workgroup reads a contiguous slice with 16-byte loads and keeps a running maximum of the words (so that
// nothing is optimised away).
__global__ __launch_bounds__(RP_BLOCK) void k_read_probe(const Vec4* __restrict__ src, i64 n_vec, unsigned* __restrict__ out)
{
    const i64 per_block = (n_vec + gridDim.x - 1) / gridDim.x;
    const i64 lo = (i64)blockIdx.x * per_block;
    i64 hi = lo + per_block;
    if (hi > n_vec) hi = n_vec;
    unsigned m = 0u;
    i64 i = lo + threadIdx.x;
    for (; i + (i64)(RP_UNROLL - 1) * RP_BLOCK < hi; i += (i64)RP_UNROLL * RP_BLOCK) {
        Vec4 v[RP_UNROLL];
#pragma unroll
        for (int k = 0; k < RP_UNROLL; ++k) v[k] = __builtin_nontemporal_load(&src[i + (i64)k * RP_BLOCK]);     // streaming hint: read once
#pragma unroll
        for (int k = 0; k < RP_UNROLL; ++k) m = max(m, max(max(v[k].x, v[k].y), max(v[k].z, v[k].w)));
    }
    for (; i < hi; i += RP_BLOCK) {
        const Vec4 v = src[i];
        m = max(m, max(max(v.x, v.y), max(v.z, v.w)));
    }
    // the words are never this value in practice; the store only keeps the reads alive (an atomic per wave on a
    // few addresses would cost more than a tenth of the pass)
    if (m == 0x7FC0DEADu) out[blockIdx.x & 63] = m;
}

}  // namespace

extern "C" int32_t disco_read_probe(const void* src, int64_t bytes, void* out64, void* stream_)
{
    if (!src || !out64) return DISCO_ERR_NULL;
    if (bytes < 0 || (bytes & 15) != 0 || ((uintptr_t)src & 15u) != 0) return DISCO_ERR_SHAPE;
    if (bytes == 0) return DISCO_OK;
    const i64 n_vec = bytes / 16;
    i64 blocks = (n_vec + (i64)RP_BLOCK * RP_UNROLL - 1) / ((i64)RP_BLOCK * RP_UNROLL);
    if (blocks > 2048) blocks = 2048;
    if (blocks < 1) blocks = 1;
    hipLaunchKernelGGL(k_read_probe, dim3((unsigned)blocks), dim3(RP_BLOCK), 0, (hipStream_t)stream_, (const Vec4*)src, n_vec,
                       (unsigned*)out64);
    DISCO_HIP(hipGetLastError());
    return DISCO_OK;
}
