// Token timelines (Sec. 4.3), general kernel: the statistics pass of tables
// the streaming kernels do not cover (it also writes the per-token deliveries
// of one column).  The histogram passes with one histogram per slot run the
// same workgroup body from the kernels of the TBT selection.
#include <string.h>

#include "disco_tl_general_kernel.h"

namespace {

__global__ __launch_bounds__(TL_BLOCK) void k_timeline(TraceView tr, i64 n_tok, int align,
                                                    const disco_policy* __restrict__ pol, TimelineArgs a)
{
    __shared__ __align__(16) unsigned smem[DISCO_TL_HIST_WORDS];
    __shared__ TimelineLds lds;
    timeline_body<false>(smem, lds, tr, n_tok, align, pol, a, blockIdx.x, gridDim.x);
}

}  // namespace

void disco_launch_timeline_general(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a,
                                   hipStream_t stream)
{
    i64 b = (v.n_req + (i64)TL_WAVES * TL_RB - 1) / ((i64)TL_WAVES * TL_RB);
    if (b < 1) b = 1;
    if (b > 512) b = 512;
    const int align = (int)(((uintptr_t)v.arr >> 2) & 3);
    hipLaunchKernelGGL(k_timeline, dim3((unsigned)b), dim3(TL_BLOCK), 0, stream, v, n_tok, align, pol, a);
}
