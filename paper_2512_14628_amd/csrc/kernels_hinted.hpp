// The projection under a predicted selection: what runs after the selection (pass 1's side is in kernels_project.hpp).
// Part of the single translation unit built from hsadmm.hip (included there, in order).
#ifndef KERNELS_HINTED_HPP
#define KERNELS_HINTED_HPP
#include "hsadmm_device.hpp"
#include "kernels_project.hpp"
#include "kernels_frozen.hpp"

namespace {

// ------------------------------------------------------------------ project under a predicted selection: repair

// After the selection every FILTER row goes from the form its prediction gave it to its final form, and the packed
// buffer is completed (`packed`: the layer's segment, or null without a compaction):
//   predicted pruned, pruned   stash: Z <- +0 (a store only; U = V is final since pass 1); else nothing to do
//   predicted pruned, kept     stash: Z holds the kept-form dual and U the candidate: the two change places;
//                              else the row is formed again from the replicas and the old dual, as pass 1 forms a
//                              row predicted kept; either way the candidate also goes to the packed row
//   predicted kept,   pruned   U <- V (held in Z), Z <- +0, as without a prediction
//   predicted kept,   kept     final; copied to the packed buffer only if its rank has changed
template <int R>
__device__ __forceinline__ void hinted_repair_rows(const WorkItem& it, const ProjectArgs& a, int Rrt,
                                                   const int32_t* __restrict__ sel_prev,
                                                   const int32_t* __restrict__ pos, bool stash, float* packed)
{
    const int row_len = it.row_len;
    const bool vec = item_vec(it);
    const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
    const int lpr = it.lpr <= kWave ? it.lpr : kBlock;
    const int rows_at_once = kBlock / lpr;
    const int sub = threadIdx.x / lpr;
    const int j = threadIdx.x - sub * lpr;
    const int nchunk = row_len >> 2;
    float* const U = a.U;
    float* const Z = a.Z;
    for (int rr = sub; rr < it.nr; rr += rows_at_once) {
        const int hp = sel_prev[it.g0 + rr];
        const int pn = pos[it.g0 + rr];
        const bool pred_kept = hp >= 0, kept = pn >= 0;
        const int64_t base = it.base + (int64_t)rr * row_len;
        float* pk = (packed && kept) ? packed + (int64_t)pn * row_len : nullptr;
        if (pred_kept && kept) {
            if (!pk || pn == hp) continue;                       // packed in pass 1 already, at this rank
            if (vec) for (int c = j; c < nchunk; c += lpr) st4u(pk + 4 * c, ld4(Z + base + 4 * c));
            else for (int c = j; c < row_len; c += lpr) pk[c] = ld1(Z + base + c);
        } else if (!pred_kept && !kept) {
            if (!stash) continue;
            if (vec) for (int c = j; c < nchunk; c += lpr) st4(Z + base + 4 * c, zero4);
            else for (int c = j; c < row_len; c += lpr) st1(Z + base + c, 0.f);
        } else if (pred_kept) {
            if (vec) {
                for (int c = j; c < nchunk; c += lpr) {
                    const int64_t e = base + 4 * c;
                    st4(U + e, ld4(Z + e));
                    st4(Z + e, zero4);
                }
            } else {
                for (int c = j; c < row_len; c += lpr) {
                    st1(U + base + c, ld1(Z + base + c));
                    st1(Z + base + c, 0.f);
                }
            }
        } else if (stash) {
            if (vec) {
                for (int c = j; c < nchunk; c += lpr) {
                    const int64_t e = base + 4 * c;
                    const v4f v = ld4(U + e), d = ld4(Z + e);
                    st4(Z + e, v);
                    st4(U + e, d);
                    if (pk) st4u(pk + 4 * c, v);
                }
            } else {
                for (int c = j; c < row_len; c += lpr) {
                    const float v = ld1(U + base + c), d = ld1(Z + base + c);
                    st1(Z + base + c, v);
                    st1(U + base + c, d);
                    if (pk) pk[c] = v;
                }
            }
        } else {
            // the same arithmetic on the same inputs as in pass 1, so the same bits (the keys are not taken again)
            if (vec) for (int c = j; c < nchunk; c += lpr) (void)Cand<R>::one_h(a, Rrt, base, c << 2, true, false, pk);
            else for (int c = j; c < row_len; c += lpr) (void)Cand<R>::scalar_h(a, Rrt, base, c, true, false, pk);
        }
    }
}

// The repair pass with the dual updated in place: every FILTER row item is visited (the rows predicted pruned and
// pruned, most of them once the pattern has settled, still hold the stashed dual in Z).
template <int R>
__global__ __launch_bounds__(kBlock) void hinted_repair_all(const WorkItem* __restrict__ fix_items, ProjectArgs a,
                                                            int Rrt, HintArgs h, PackOut po)
{
    const WorkItem it = fix_items[blockIdx.x];
    hinted_repair_rows<R>(it, a, Rrt, h.sel_prev, po.pos, true, po.packed ? po.packed + it.packed_off : nullptr);
}

// The repair pass with the dual written out of place: a fixed number of workgroups share the row items the
// selection has listed (none at all when the prediction was right everywhere).  A listed item of a CHANNEL layer
// belongs to a layer whose kept channels are not the predicted ones: its rows are formed again under the mask
// just selected, from the replicas and the old dual (the frozen-mask pass).
template <int R>
__global__ __launch_bounds__(kBlock) void hinted_repair(const WorkItem* __restrict__ row_items, ProjectArgs a, int Rrt,
                                                        HintArgs h, const uint8_t* __restrict__ mask, PackOut po)
{
    const int n = h.work[0];
    for (int i = blockIdx.x; i < n; i += gridDim.x) {
        const WorkItem it = row_items[h.work[kWorkHeader + i]];
        if (item_mode(it) == HSADMM_MODE_CHANNEL) {
            if (po.packed) frozen_item<R, true>(it, a, Rrt, mask, po);
            else frozen_item<R, false>(it, a, Rrt, mask, po);
        } else {
            hinted_repair_rows<R>(it, a, Rrt, h.sel_prev, po.pos, false, po.packed ? po.packed + it.packed_off : nullptr);
        }
    }
}

}  // namespace
#endif
