// One class-mode TBT histogram pass over the timelines with a buffer hand-off
// (Sec. 4.3) that have tokens to walk: the workgroup body, shared by the
// kernel of the regular passes and the kernel of the spare passes.
#pragma once
#include "disco_tl_general.h"
#include "disco_tl_walk.h"

namespace {

constexpr int TBH_BLOCK = 1024;              // histogram workgroups: 16 waves share the LDS bins

struct BufHistArgs {
    HistArgs h;
    BufCostArgs bc;
    const unsigned* buffer_flag;
};

// Workgroup `bid` of `nblk`: bytes 3 and 4 of a request's descriptor name the LDS rows of its two hand-off kinds,
// the walk list of the selection names the requests.  `smem`: DISCO_TL_HIST_WORDS words of LDS.
__device__ __forceinline__ void tl_hist_buf_body(unsigned* smem, const TraceView& tr, i64 n_tok, int align, const BufHistArgs& ba,
                                                 unsigned bid, unsigned nblk)
{
    const HistArgs& a = ba.h;
    const TlSel* tl = &a.S->tl;
    const int width = tl->width;
    if (*ba.buffer_flag == 0u || width <= 0 || tl->fallback) return;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int ncls = tl->ncls, nwalk = tl->nwalk;
    HistCtx h;
    h.hist = smem; h.width = width; h.shift = tl->shift; h.up = h.shift + width;
    h.G = tl->G < DISCO_MAX_GRP ? tl->G : DISCO_MAX_GRP;
    h.stride = (unsigned)nwalk << width;
    h.key_lo = tl->key_lo; h.key_cap = tl->window ? (1u << tl->window) : 0xFFFFFFFFu;
    for (int k = 0; k < DISCO_MAX_GRP; ++k) h.grp_prefix[k] = tl->grp_prefix[k];
    const int words = (h.G * nwalk) << width;
    for (int i = threadIdx.x; i < words; i += TBH_BLOCK) smem[i] = 0u;
    __syncthreads();
    const i64 nwaves = (i64)nblk * (TBH_BLOCK / 64);
    const i64 nfront = (i64)tl->nlist, nlist = nfront + (i64)tl->nlist_back;
    i64 rb = (nlist + nwaves - 1) / nwaves;
    rb = rb < 1 ? 1 : (rb > 64 ? 64 : rb);
    const i64 nround = (nlist + rb * nwaves - 1) / (rb * nwaves);
    for (i64 rnd = 0; rnd < nround; ++rnd) {
        const i64 gw = (i64)bid * (TBH_BLOCK / 64) + wave;
        const i64 j = rnd * rb * nwaves + gw + (i64)lane * nwaves;
        const bool mine = lane < rb && j < nlist;
        const i64 il = mine ? (i64)walk_list_entry(a.list, tr.n_req, nfront, j) : 0;
        const unsigned desc = mine ? (unsigned)((a.desc[il] >> 24) & 0xFFFFull) : 0xFFFFu;
        u64 walkers = __ballot(desc != 0xFFFFu);
        if (!walkers) continue;
        int l_v = 0, n_v = 1;
        float k_v = tr.k_s, gd_v = tr.g_s, gap_v = 0.0f, s_v = 0.0f;
        i64 off_v = 0;
        if (desc != 0xFFFFu) {
            l_v = tr.l[il]; n_v = tr.n[il]; s_v = tr.s[il];
            if (tr.k) k_v = tr.k[il];
            if (tr.g) gd_v = tr.g[il];
            if (tr.off) off_v = tr.off[il];
            if (tr.tbt) gap_v = tr.tbt[il];
        }
        while (walkers) {
            const int rq = __ffsll((long long)walkers) - 1;
            walkers &= walkers - 1;
            const unsigned dsc = (unsigned)bcast_i((int)desc, rq);
            const int n = bcast_i(n_v, rq), l = bcast_i(l_v, rq);
            const float k = bcast_f(k_v, rq), gd = bcast_f(gd_v, rq), gap = bcast_f(gap_v, rq), s_ttft = bcast_f(s_v, rq);
            const i64 off = tr.arr ? (i64)bcast_u64((u64)off_v, rq) : 0;
#pragma unroll 1
            for (int kind = 1; kind >= 0; --kind) {
                const unsigned sl = (dsc >> (8 * kind)) & 0xFFu;
                if (sl == 0xFFu) continue;
                const unsigned row_base = sl << width;
                auto sink = [&](const unsigned key[4], const bool ok[4]) {
                    const unsigned kk[4] = {ok[0] ? key[0] : KEY_SKIP, ok[1] ? key[1] : KEY_SKIP, ok[2] ? key[2] : KEY_SKIP,
                                            ok[3] ? key[3] : KEY_SKIP};
                    hist_keys(h, kk, row_base, lane);
                };
                (void)run_timeline(TL_SRV_BUF + kind, n, tr.arr, off, n_tok, align, gap, gd, l, k, tr.c, s_ttft, ba.bc, a.tau, a.kt,
                                   lane, nullptr, sink);
            }
        }
    }
    __syncthreads();
    // LDS rows (group, walked class) -> device-wide rows (group, class)
    const unsigned dmask = (1u << width) - 1u;
    for (int i = threadIdx.x; i < words; i += TBH_BLOCK) {
        const unsigned cnt = smem[i];
        if (!cnt) continue;
        const int row = i >> width;
        const int g = row / nwalk, sl = row - g * nwalk;
        const int c = tl->slot_cls[sl];
        atomicAdd(&a.ghist[((size_t)(g * ncls + c) << width) | ((unsigned)i & dmask)], cnt);
    }
}

}  // namespace
