// Host-side launch interface between the translation units of libdisco.
#pragma once
#include "disco_state.h"

struct TimelineArgs {
    float tau, kt;            // pacing interval, kappa_lag * tau
    int P, nq, pass;          // pass < 0: statistics pass, else histogram pass `pass` of the TBT selection
    int32_t* mig_idx; int32_t* n_src_tok; float* t_last; float* delivered; int delivered_col;
    MigPartial* part; unsigned* ticket; disco_accum* acc;
    SelState* S; unsigned* ghist;
};

SelPlan disco_tbt_plan(int P, int nq);
void disco_launch_timeline(const TraceView& v, i64 n_tok, const disco_policy* pol, const TimelineArgs& a,
                           hipStream_t stream);
