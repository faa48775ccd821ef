// The projection under a predicted selection: pass 1 of the layers under both constraints, the pass-1 kernel, and
// what runs after the selection (pass 1's side for the other modes is in kernels_project.hpp).
// Part of the single translation unit built from hsadmm.hip (included there, in order).
#ifndef KERNELS_HINTED_HPP
#define KERNELS_HINTED_HPP
#include "hsadmm_device.hpp"
#include "kernels_project.hpp"
#include "kernels_frozen.hpp"

namespace {

// ------------------------------------------------------------------ layers under both constraints, predicted

// For 4 adjacent columns of a layer under both constraints: whether the record predicts the column's channel kept,
// and the column's place in a packed row (-1: none; a rank outside [0, k_in) cannot have come from a selection of
// this plan and is never used as an address).  rank: the channel part of the layer's record.
__device__ __forceinline__ void quad_predicted_cols(const int32_t* __restrict__ rank, const DivKhw& div, int col,
                                                    int k_in, bool kept[4], int pc[4])
{
    if (div.khw == 1) {
        int4 r;
        __builtin_memcpy(&r, rank + col, 16);
        const int rr[4] = {r.x, r.y, r.z, r.w};
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            kept[i] = rr[i] >= 0;
            pc[i] = (rr[i] >= 0 && rr[i] < k_in) ? rr[i] : -1;
        }
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int ch = div(col + i);
            const int r = rank[ch];
            kept[i] = r >= 0;
            pc[i] = (r >= 0 && r < k_in) ? r * div.khw + (col + i - ch * div.khw) : -1;
        }
    }
}

// The outputs of 4 adjacent elements of a layer under both constraints in the form the two predicted selections make
// final: kept (its filter and its channel are predicted kept) Z <- V, else Z <- +0; U + (Wbar - Z) to the new dual;
// a kept element of a row that is packed (drow) also to its packed column (vd: the inter-node dual that is added to
// what is packed when the candidate is the weighted one; unused otherwise: z is packed bit for bit).
template <bool WEIGHTED>
__device__ __forceinline__ void both_put(const ProjectArgs& a, int64_t e, const v4f& wb, const v4f& u, const v4f& v,
                                         const v4f& vd, bool row_kept, const bool kept[4], const int pc[4], float* drow)
{
    v4f z;
    z.x = (row_kept && kept[0]) ? v.x : 0.f;
    z.y = (row_kept && kept[1]) ? v.y : 0.f;
    z.z = (row_kept && kept[2]) ? v.z : 0.f;
    z.w = (row_kept && kept[3]) ? v.w : 0.f;
    st4(a.Z + e, z);
    st4(a.U + e, u + (wb - z));
    if (a.Wbar) st4(a.Wbar + e, wb);
    if (drow) {
        const v4f c = WEIGHTED ? z + vd : z;
        if (pc[0] >= 0) drow[pc[0]] = c.x;
        if (pc[1] >= 0) drow[pc[1]] = c.y;
        if (pc[2] >= 0) drow[pc[2]] = c.z;
        if (pc[3] >= 0) drow[pc[3]] = c.w;
    }
}

// The candidate of 4 adjacent elements from the mean and the old dual: Wbar + U, or (WEIGHTED) Eq. (9)'s
// z~ = fl(fl(a t) + fl(b (Zg - Vd))), t = Wbar + U, with the arithmetic of the un-predicted weighted pass; vd: Vd.
template <bool WEIGHTED>
__device__ __forceinline__ v4f both_candidate(const ProjectArgs& a, int64_t e, const v4f& wb, const v4f& u, float al,
                                              float bl, v4f& vd)
{
    v4f v = wb + u;
    vd = v4f{0.f, 0.f, 0.f, 0.f};
    if (WEIGHTED) {
        vd = ld4(a.Vd + e);
        const v4f q = ld4(a.Zg + e) - vd;
        const v4f at = v * al;
        const v4f bq = q * bl;
        v = at + bq;
    }
    return v;
}

// pass1_row<R, true> (the row's share of its filter norm: squares of the whole candidate row, same chunks, same
// order) with the row written in its predicted final form instead of the parked mean.
template <int R, bool WEIGHTED>
__device__ __forceinline__ double pass1_row_both_hinted(const ProjectArgs& a, int Rrt, int64_t base, int row_len,
                                                        bool vec, int j, int step, bool row_kept,
                                                        const int32_t* __restrict__ hp_c, const DivKhw& div, int k_in,
                                                        float* drow, float al, float bl)
{
    const int RR = R > 0 ? R : Rrt;
    double acc = 0.0;
    if (vec) {
        const int nchunk = row_len >> 2;
        int c = j;
        for (; c + step < nchunk; c += 2 * step) {
            const int col0 = c << 2, col1 = (c + step) << 2;
            const int64_t e0 = base + col0, e1 = base + col1;
            v4f s0 = ld4(a.W[0] + e0), s1 = ld4(a.W[0] + e1);
#pragma unroll
            for (int r = 1; r < RR; ++r) {
                const v4f w0 = ld4(a.W[r] + e0), w1 = ld4(a.W[r] + e1);
                s0 = s0 + w0;
                s1 = s1 + w1;
            }
            const v4f u0 = ld4(a.Ur + e0), u1 = ld4(a.Ur + e1);
            bool k0[4], k1[4];
            int p0[4], p1[4];
            quad_predicted_cols(hp_c, div, col0, k_in, k0, p0);
            quad_predicted_cols(hp_c, div, col1, k_in, k1, p1);
            const v4f wb0 = s0 * a.inv_R, wb1 = s1 * a.inv_R;
            v4f vd0, vd1;
            const v4f v0 = both_candidate<WEIGHTED>(a, e0, wb0, u0, al, bl, vd0);
            const v4f v1 = both_candidate<WEIGHTED>(a, e1, wb1, u1, al, bl, vd1);
            both_put<WEIGHTED>(a, e0, wb0, u0, v0, vd0, row_kept, k0, p0, drow);
            both_put<WEIGHTED>(a, e1, wb1, u1, v1, vd1, row_kept, k1, p1, drow);
            acc = sq4(acc, v0);
            acc = sq4(acc, v1);
        }
        if (c < nchunk) {
            const int col = c << 2;
            const int64_t e = base + col;
            v4f s = ld4(a.W[0] + e);
#pragma unroll
            for (int r = 1; r < RR; ++r) s = s + ld4(a.W[r] + e);
            const v4f u = ld4(a.Ur + e);
            bool k[4];
            int p[4];
            quad_predicted_cols(hp_c, div, col, k_in, k, p);
            const v4f wb = s * a.inv_R;
            v4f vd;
            const v4f v = both_candidate<WEIGHTED>(a, e, wb, u, al, bl, vd);
            both_put<WEIGHTED>(a, e, wb, u, v, vd, row_kept, k, p, drow);
            acc = sq4(acc, v);
        }
    } else {
        for (int c = j; c < row_len; c += step) {
            const int64_t e = base + c;
            float s = ld1(a.W[0] + e);
            for (int r = 1; r < RR; ++r) s = s + ld1(a.W[r] + e);
            const float u = ld1(a.Ur + e);
            const float wb = s * a.inv_R;
            float v = wb + u;
            float vd = 0.f;
            if (WEIGHTED) {
                vd = ld1(a.Vd + e);
                const float q = ld1(a.Zg + e) - vd;
                const float at = v * al;
                const float bq = q * bl;
                v = at + bq;
            }
            const int ch = div(c);
            const int r = hp_c[ch];
            const float z = (row_kept && r >= 0) ? v : 0.f;
            st1(a.Z + e, z);
            st1(a.U + e, u + (wb - z));
            if (a.Wbar) st1(a.Wbar + e, wb);
            if (drow && r >= 0 && r < k_in) drow[r * div.khw + (c - ch * div.khw)] = WEIGHTED ? z + vd : z;
            acc = fma((double)v, (double)v, acc);
        }
    }
    return acc;
}

// project_rows<R, true> (row items of a layer under both constraints) under a predicted selection, for a dual written
// out of place: the filter norms as there, and instead of the parked mean the layer's outputs in the form the record
// makes final -- an element is kept if its filter and its channel are predicted kept; rows predicted kept at a rank
// in [0, k) also go to the packed buffer, their kept columns at the predicted packed columns.  The channel norms of
// the second selection are then taken from these outputs (composite_colsums_hinted); if both selections turn out as
// predicted the layer is done, else the repair pass forms it again from the replicas and the old dual.
// WEIGHTED: the candidate of Eq. (9) (its norms, and c = z + Vd packed), see both_candidate.
template <int R, bool WEIGHTED = false>
__device__ __forceinline__ void project_rows_both_hinted(const WorkItem& it, const ProjectArgs& a, int Rrt,
                                                         const HintArgs& h)
{
    const float al = WEIGHTED ? a.coef[2 * it.layer] : 1.f, bl = WEIGHTED ? a.coef[2 * it.layer + 1] : 0.f;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = it.row_len;
    const bool vec = item_vec(it);
    const DivKhw div(it.khw);
    const int k_in = h.layers[it.layer].k_in;
    const int packed_row_len = k_in * it.khw;
    const int32_t* hp_c = h.sel_prev + it.aux;                   // the channel part of the layer's record
    float* const pk_layer = h.packed ? h.packed + it.packed_off : nullptr;
    auto prediction = [&](int rr, bool& kept, float*& drow) {
        const int hp = h.sel_prev[it.g0 + rr];
        kept = hp >= 0;
        drow = (pk_layer && kept && hp < it.k) ? pk_layer + (int64_t)hp * packed_row_len : nullptr;
    };
    if (it.lpr <= kWave) {
        const int lpr = it.lpr;
        const int rpw = kWave / lpr;
        const int sub = lane / lpr;
        const int j = lane - sub * lpr;
        for (int rb = wave * rpw; rb < it.nr; rb += kWaves * rpw) {
            const int rr = rb + sub;
            const bool active = rr < it.nr;
            double acc = 0.0;
            if (active) {
                bool kept;
                float* drow;
                prediction(rr, kept, drow);
                acc = pass1_row_both_hinted<R, WEIGHTED>(a, Rrt, it.base + (int64_t)rr * row_len, row_len, vec, j, lpr,
                                                         kept, hp_c, div, k_in, drow, al, bl);
            }
            acc = wave_xor_sum(acc, lpr);
            if (active && j == 0) a.key[it.g0 + rr] = acc;
        }
    } else {
        __shared__ double wsum[kWaves];
        for (int rr = 0; rr < it.nr; ++rr) {
            bool kept;
            float* drow;
            prediction(rr, kept, drow);
            double acc = pass1_row_both_hinted<R, WEIGHTED>(a, Rrt, it.base + (int64_t)rr * row_len, row_len, vec,
                                                            threadIdx.x, kBlock, kept, hp_c, div, k_in, drow, al, bl);
            acc = wave_xor_sum(acc, kWave);
            if (lane == 0) wsum[wave] = acc;
            __syncthreads();
            if (threadIdx.x == 0) {
                double s = wsum[0];
                for (int w = 1; w < kWaves; ++w) s += wsum[w];
                a.key[it.g0 + rr] = s;
            }
            __syncthreads();
        }
    }
}

// composite_colsums for layers that pass 1 wrote under a prediction: the candidate of a kept filter's row is read
// back from the outputs -- Z where the element was predicted kept, the new dual where it was not (a pruned element's
// dual is U + Wbar, the candidate bit for bit) -- whatever the filter selection turned out to be.  Tiles and the
// order of additions are those of composite_colsums.  With coef (the weighted candidate of Eq. (9)) a pruned
// element's dual is t = Wbar + U and its candidate is formed again as fl(fl(a t) + fl(b (Zg - Vd))).
__global__ __launch_bounds__(kBlock) void composite_colsums_hinted(const WorkItem* __restrict__ items,
                                                                   const DevLayer* __restrict__ layers,
                                                                   const float* __restrict__ Z,
                                                                   const float* __restrict__ Unew,
                                                                   const float* __restrict__ Zg,
                                                                   const float* __restrict__ Vd,
                                                                   const float* __restrict__ coef,
                                                                   const int32_t* __restrict__ sel_prev,
                                                                   const uint8_t* __restrict__ mask,
                                                                   double* __restrict__ colpart)
{
    __shared__ double part[kWaves][kWave * 4];
    const WorkItem it = items[blockIdx.x];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = it.row_len;
    const bool vec = item_vec(it);
    const int vw = vec ? 4 : 1;
    const int col = it.col0 + lane * vw;
    const bool in = col < row_len;
    const uint8_t* mf = mask + it.g0 + it.row0;                  // filter bytes of the tile's rows
    const int32_t* hp_f = sel_prev + it.g0 + it.row0;            // ... and their predictions
    const int32_t* hp_c = sel_prev + it.g0 + layers[it.layer].c_out;
    const float al = coef ? coef[2 * it.layer] : 1.f, bl = coef ? coef[2 * it.layer + 1] : 0.f;
    double acc0 = 0.0, acc1 = 0.0, acc2 = 0.0, acc3 = 0.0;
    if (in) {
        const DivKhw div(it.khw);
        bool ck[4] = {false, false, false, false};
#pragma unroll
        for (int i = 0; i < 4; ++i)
            if (i < vw) ck[i] = hp_c[div(col + i)] >= 0;
        for (int rr = wave; rr < it.nr; rr += kWaves) {
            if (mf[rr] == 0) continue;
            const bool rk = hp_f[rr] >= 0;
            const int64_t e = it.base + (int64_t)rr * row_len + col;
            if (vec) {
                const v4f z = ld4(Z + e);
                v4f u = ld4(Unew + e);
                if (coef) {
                    const v4f q = ld4(Zg + e) - ld4(Vd + e);
                    const v4f at = u * al;
                    const v4f bq = q * bl;
                    u = at + bq;
                }
                v4f v;
                v.x = (rk && ck[0]) ? z.x : u.x;
                v.y = (rk && ck[1]) ? z.y : u.y;
                v.z = (rk && ck[2]) ? z.z : u.z;
                v.w = (rk && ck[3]) ? z.w : u.w;
                acc0 = fma((double)v.x, (double)v.x, acc0);
                acc1 = fma((double)v.y, (double)v.y, acc1);
                acc2 = fma((double)v.z, (double)v.z, acc2);
                acc3 = fma((double)v.w, (double)v.w, acc3);
            } else {
                float u = ld1(Unew + e);
                if (coef) {
                    const float q = ld1(Zg + e) - ld1(Vd + e);
                    const float at = u * al;
                    const float bq = q * bl;
                    u = at + bq;
                }
                const float v = (rk && ck[0]) ? ld1(Z + e) : u;
                acc0 = fma((double)v, (double)v, acc0);
            }
        }
    }
    part[wave][lane * 4 + 0] = acc0;
    part[wave][lane * 4 + 1] = acc1;
    part[wave][lane * 4 + 2] = acc2;
    part[wave][lane * 4 + 3] = acc3;
    __syncthreads();
    if (wave == 0 && in) {
        double* out = colpart + it.aux + col;
        for (int i = 0; i < vw; ++i) {
            double s = part[0][lane * 4 + i];
            for (int w = 1; w < kWaves; ++w) s += part[w][lane * 4 + i];
            out[i] = s;
        }
    }
}

// Pass 1 under a predicted selection: FILTER and NONE layers by project_rows_hinted.  CHANNEL and BOTH layers take
// the prediction when the dual is written out of place (TILES: an instantiation of its own for plans with such layers,
// so that the other plans' kernel keeps its registers); else they only sum here and are written after the selection.
template <int R, bool TILES = false>
__global__ __launch_bounds__(kBlock) void project_pass1_hinted(const WorkItem* __restrict__ items, ProjectArgs a,
                                                               int Rrt, HintArgs h)
{
    const WorkItem it = items[blockIdx.x];
    const int mode = item_mode(it);
    if (blockIdx.x == 0 && threadIdx.x == 0) h.work[0] = 0;      // (the selection runs after this whole launch)
    if (mode == HSADMM_MODE_CHANNEL) {
        if constexpr (TILES) project_tile_hinted<R>(it, a, Rrt, h);
        else project_tile<R>(it, a, Rrt);
    } else if (mode == HSADMM_MODE_BOTH) {
        if constexpr (TILES) project_rows_both_hinted<R>(it, a, Rrt, h);
        else project_rows<R, true>(it, a, Rrt);
    } else {
        project_rows_hinted<R>(it, a, Rrt, h);
    }
}

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
// selection has listed (none at all when the prediction was right everywhere).  A listed item of a CHANNEL or BOTH
// layer belongs to a layer whose kept groups are not the predicted ones: its rows are formed again under the mask
// just selected, from the replicas and the old dual (the frozen-mask pass).
template <int R>
__global__ __launch_bounds__(kBlock) void hinted_repair(const WorkItem* __restrict__ row_items, ProjectArgs a, int Rrt,
                                                        HintArgs h, const uint8_t* __restrict__ mask, PackOut po)
{
    const int n = h.work[0];
    for (int i = blockIdx.x; i < n; i += gridDim.x) {
        const WorkItem it = row_items[h.work[kWorkHeader + i]];
        if (mode_has_channels(item_mode(it))) {
            if (po.packed) frozen_item<R, true>(it, a, Rrt, mask, po);
            else frozen_item<R, false>(it, a, Rrt, mask, po);
        } else {
            hinted_repair_rows<R>(it, a, Rrt, h.sel_prev, po.pos, false, po.packed ? po.packed + it.packed_off : nullptr);
        }
    }
}

}  // namespace
#endif
