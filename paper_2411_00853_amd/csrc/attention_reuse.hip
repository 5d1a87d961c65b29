// The attention chunk kernel with ordinary (cached) loads of the keys and values: for launches in which
// several work items stream the same cache head (see attention_kernel.h).
#include "attention_kernel.h"

namespace specv {

int launch_chunks_reuse(int hd, int rt, int cw, dim3 grid, dim3 wg_grid, hipStream_t s, const StepTables& t,
                        const LookaheadPack& ks, const CacheGeom& g, int n_q_heads, int kv_share, int layer, const void* cache,
                        const float* q, const AttnPlan& p, int r_cap, float sl2, float* part_o, float* part_ml,
                        const QkvSrc& src, void* cache_w, const XOut& xo)
{
    if (hd == 64)
        return launch_chunks<64, false>(rt, cw, grid, wg_grid, s, t, ks, g, n_q_heads, kv_share, layer, cache, q, p, r_cap, sl2,
                                        part_o, part_ml, src, cache_w, xo);
    return launch_chunks<128, false>(rt, cw, grid, wg_grid, s, t, ks, g, n_q_heads, kv_share, layer, cache, q, p, r_cap, sl2,
                                     part_o, part_ml, src, cache_w, xo);
}

}  // namespace specv
