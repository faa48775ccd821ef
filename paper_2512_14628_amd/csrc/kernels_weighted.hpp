// hsadmm_project_weighted (full candidate of Eq. (9)), hsadmm_dual_inter (Eq. (13)) and hsadmm_average (Eq. (11)).
// Part of the single translation unit built from hsadmm.hip (included there, in order).
#ifndef KERNELS_WEIGHTED_HPP
#define KERNELS_WEIGHTED_HPP
#include "hsadmm_device.hpp"

namespace {

// ------------------------------------------------------------------ full node update (Eq. (9)) and Eq. (13)

struct WeightedArgs {
    ProjectArgs p;
    const float* Zg;      // global consensus z
    const float* Vd;      // inter-node dual v_i
    const float* coef;    // per layer: a_l, b_l
    // weighted_pass1<R, true> (the pass that also takes the intra-node residual sums of Section 3.4):
    const float* Zi_prev; // the previous z_i, a buffer other than Z
    double* rowres;       // 4 doubles per group of the FILTER and unconstrained layers, see weighted_pass1
};

// z~ = fl(fl(a t) + fl(b q)) with t = Wbar + U, q = z - v, for 4 (or 1) adjacent elements; no stores.
template <int R>
__device__ __forceinline__ void wcand4(const WeightedArgs& w, int Rrt, int64_t e, float al, float bl,
                                       v4f& wb, v4f& u, v4f& zt)
{
    const int RR = R > 0 ? R : Rrt;
    v4f s = ld4(w.p.W[0] + e);
#pragma unroll
    for (int r = 1; r < RR; ++r) s = s + ld4(w.p.W[r] + e);
    u = ld4(w.p.Ur + e);
    const v4f q = ld4(w.Zg + e) - ld4(w.Vd + e);
    wb = s * w.p.inv_R;
    const v4f t = wb + u;
    const v4f at = t * al;
    const v4f bq = q * bl;
    zt = at + bq;
}

// the same for two chunks, with every load issued before any arithmetic
template <int R>
__device__ __forceinline__ void wcand4x2(const WeightedArgs& w, int Rrt, int64_t e0, int64_t e1, float al, float bl,
                                         v4f& wb0, v4f& u0, v4f& zt0, v4f& wb1, v4f& u1, v4f& zt1)
{
    const int RR = R > 0 ? R : Rrt;
    v4f s0 = ld4(w.p.W[0] + e0), s1 = ld4(w.p.W[0] + e1);
#pragma unroll
    for (int r = 1; r < RR; ++r) {
        const v4f x0 = ld4(w.p.W[r] + e0), x1 = ld4(w.p.W[r] + e1);
        s0 = s0 + x0;
        s1 = s1 + x1;
    }
    u0 = ld4(w.p.Ur + e0);
    u1 = ld4(w.p.Ur + e1);
    const v4f g0 = ld4(w.Zg + e0), g1 = ld4(w.Zg + e1);
    const v4f d0 = ld4(w.Vd + e0), d1 = ld4(w.Vd + e1);
    const v4f q0 = g0 - d0, q1 = g1 - d1;
    wb0 = s0 * w.p.inv_R;
    wb1 = s1 * w.p.inv_R;
    const v4f t0 = wb0 + u0, t1 = wb1 + u1;
    const v4f at0 = t0 * al, at1 = t1 * al;
    const v4f bq0 = q0 * bl, bq1 = q1 * bl;
    zt0 = at0 + bq0;
    zt1 = at1 + bq1;
}

// wcand4 that also adds the element's terms of the intra-node residual sums for either outcome of its row:
//   acc[0] += sum_j (W_j - z~)^2   acc[2] += (z~ - z_prev)^2      if the row is kept (z_i = z~)
//   acc[1] += sum_j W_j^2          acc[3] += z_prev^2             if it is pruned (z_i = 0)
// in fp64 from the fp32 values.  With a compile-time R the replicas' values stay in registers, else they are read
// a second time.
template <int R>
__device__ __forceinline__ void wcand4_res(const WeightedArgs& w, int Rrt, int64_t e, float al, float bl,
                                           v4f& wb, v4f& u, v4f& zt, v4f& vd, double acc[4])
{
    const int RR = R > 0 ? R : Rrt;
    constexpr int kHeld = R > 0 ? R : 1;
    const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
    v4f held[kHeld];
    v4f s = ld4(w.p.W[0] + e);
    if (R > 0) held[0] = s;
#pragma unroll
    for (int r = 1; r < RR; ++r) {
        const v4f x = ld4(w.p.W[r] + e);
        if (R > 0) held[r] = x;
        s = s + x;
    }
    u = ld4(w.p.Ur + e);
    vd = ld4(w.Vd + e);
    const v4f q = ld4(w.Zg + e) - vd;
    const v4f zp = ld4(w.Zi_prev + e);
    wb = s * w.p.inv_R;
    const v4f t = wb + u;
    const v4f at = t * al;
    const v4f bq = q * bl;
    zt = at + bq;
#pragma unroll
    for (int r = 0; r < RR; ++r) {
        const v4f x = R > 0 ? held[r] : ld4(w.p.W[r] + e);
        acc[0] = sqd4(acc[0], x, zt);
        acc[1] = sqd4(acc[1], x, zero4);
    }
    acc[2] = sqd4(acc[2], zt, zp);
    acc[3] = sqd4(acc[3], zero4, zp);
}

template <int R>
__device__ __forceinline__ void wcand1_res(const WeightedArgs& w, int Rrt, int64_t e, float al, float bl,
                                           float& wb, float& u, float& zt, float& vd, double acc[4])
{
    const int RR = R > 0 ? R : Rrt;
    float s = ld1(w.p.W[0] + e);
    for (int r = 1; r < RR; ++r) s = s + ld1(w.p.W[r] + e);
    u = ld1(w.p.Ur + e);
    vd = ld1(w.Vd + e);
    const float q = ld1(w.Zg + e) - vd;
    const float zp = ld1(w.Zi_prev + e);
    wb = s * w.p.inv_R;
    const float t = wb + u;
    const float at = t * al;
    const float bq = q * bl;
    zt = at + bq;
    for (int r = 0; r < RR; ++r) {
        const float x = ld1(w.p.W[r] + e);
        acc[0] = sqd(acc[0], x, zt);
        acc[1] = sqd(acc[1], x, 0.f);
    }
    acc[2] = sqd(acc[2], zt, zp);
    acc[3] = sqd(acc[3], 0.f, zp);
}

template <int R>
__device__ __forceinline__ void wcand1(const WeightedArgs& w, int Rrt, int64_t e, float al, float bl,
                                       float& wb, float& u, float& zt)
{
    const int RR = R > 0 ? R : Rrt;
    float s = ld1(w.p.W[0] + e);
#pragma unroll
    for (int r = 1; r < RR; ++r) s = s + ld1(w.p.W[r] + e);
    u = ld1(w.p.Ur + e);
    const float q = ld1(w.Zg + e) - ld1(w.Vd + e);
    wb = s * w.p.inv_R;
    const float t = wb + u;
    const float at = t * al;
    const float bq = q * bl;
    zt = at + bq;
}

// Pass 1 of the weighted projection: keys of the candidate z~ with the lane mappings and the order of
// additions of project_pass1.  With the rho_2 term a pruned group needs t = Wbar + U (its dual becomes t) and
// a kept group z~ and U + (Wbar - z~); z~ follows from t, Zg and Vd, so per mode:
//   FILTER   Z <- t (a stash), U <- U + (Wbar - z~) (final if kept); weighted_fixup finishes either case
//            without reading the replicas again;
//   NONE     everything is kept: Z <- z~ and U are final;
//   BOTH     the filter norms of z~; the mean Wbar is parked in Z and U is left alone: composite_colsums and the
//            final pass (the frozen-mask kernel in its weighted form) form z~ again from Z, U, Zg and Vd;
//   CHANNEL  partial column sums; with 3 or more replicas the mean is parked in Z for the final pass.
// RES: the pass also takes, per row of a FILTER or unconstrained layer, the row's share of the intra-node residual
// sums of Section 3.4 for either outcome of the row (see wcand4_res) and leaves them in rowres[4 * group ..]; after
// the selection select_topk adds up, per layer, the sums of the outcome every row got.  The previous z_i is read
// from a buffer of its own (Z receives the stash).  CHANNEL and BOTH layers take no part in this here: their sums
// come from a pass over their final values (residual_partials on their row items).
template <int R, bool RES = false>
__device__ __forceinline__ void weighted_item(const WorkItem& it, const WeightedArgs& w, int Rrt)
{
    __shared__ double wsum[kWaves][5];
    __shared__ double part[kWaves][kWave * 4];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = it.row_len;
    const bool vec = item_vec(it);
    const float al = w.coef[2 * it.layer], bl = w.coef[2 * it.layer + 1];
    if (item_mode(it) != HSADMM_MODE_CHANNEL) {
        const int mode = item_mode(it);
        const bool park = mode == HSADMM_MODE_BOTH;
        const bool all_kept = mode == HSADMM_MODE_NONE;
        const bool wide = it.lpr > kWave;
        const int lpr = wide ? kBlock : it.lpr;
        const int rows_at_once = kBlock / lpr;
        const int sub = threadIdx.x / lpr;
        const int j = threadIdx.x - sub * lpr;
        const int rounds = (it.nr + rows_at_once - 1) / rows_at_once;
        for (int rd = 0; rd < rounds; ++rd) {
            const int rr = rd * rows_at_once + sub;
            const bool active = rr < it.nr;
            const int64_t base = it.base + (int64_t)rr * row_len;
            double acc = 0.0;
            double res[4] = {0.0, 0.0, 0.0, 0.0};
            const bool take_res = RES && !park;
            if (active) {
                if (vec) {
                    const int nchunk = row_len >> 2;
                    int c = j;
                    // two chunks of the row at a time: all their loads are issued before the first store
                    // (one at a time when the residual sums are taken: the replicas' values stay live then)
                    for (; !take_res && c + lpr < nchunk; c += 2 * lpr) {
                        const int64_t e0 = base + ((int64_t)c << 2), e1 = base + ((int64_t)(c + lpr) << 2);
                        v4f wb0, u0, zt0, wb1, u1, zt1;
                        wcand4x2<R>(w, Rrt, e0, e1, al, bl, wb0, u0, zt0, wb1, u1, zt1);
                        if (park) {
                            st4(w.p.Z + e0, wb0);
                            st4(w.p.Z + e1, wb1);
                        } else {
                            st4(w.p.Z + e0, all_kept ? zt0 : wb0 + u0);
                            st4(w.p.Z + e1, all_kept ? zt1 : wb1 + u1);
                            st4(w.p.U + e0, u0 + (wb0 - zt0));
                            st4(w.p.U + e1, u1 + (wb1 - zt1));
                            if (w.p.Wbar) { st4(w.p.Wbar + e0, wb0); st4(w.p.Wbar + e1, wb1); }
                        }
                        acc = sq4(acc, zt0);
                        acc = sq4(acc, zt1);
                    }
                    for (; c < nchunk; c += lpr) {
                        v4f wb, u, zt, vd;
                        const int64_t e = base + ((int64_t)c << 2);
                        if (take_res) wcand4_res<R>(w, Rrt, e, al, bl, wb, u, zt, vd, res);
                        else wcand4<R>(w, Rrt, e, al, bl, wb, u, zt);
                        if (park) {
                            st4(w.p.Z + e, wb);
                        } else {
                            st4(w.p.Z + e, all_kept ? zt : wb + u);
                            st4(w.p.U + e, u + (wb - zt));
                            if (w.p.Wbar) st4(w.p.Wbar + e, wb);
                        }
                        acc = sq4(acc, zt);
                    }
                } else {
                    for (int c = j; c < row_len; c += lpr) {
                        float wb, u, zt, vd;
                        if (take_res) wcand1_res<R>(w, Rrt, base + c, al, bl, wb, u, zt, vd, res);
                        else wcand1<R>(w, Rrt, base + c, al, bl, wb, u, zt);
                        if (park) {
                            st1(w.p.Z + base + c, wb);
                        } else {
                            st1(w.p.Z + base + c, all_kept ? zt : wb + u);
                            st1(w.p.U + base + c, u + (wb - zt));
                            if (w.p.Wbar) st1(w.p.Wbar + base + c, wb);
                        }
                        acc = fma((double)zt, (double)zt, acc);
                    }
                }
            }
            if (!wide) {
                acc = wave_xor_sum(acc, lpr);
                if (active && j == 0) w.p.key[it.g0 + rr] = acc;
                if (take_res) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        res[k] = wave_xor_sum(res[k], lpr);
                        if (active && j == 0) w.rowres[4 * (int64_t)(it.g0 + rr) + k] = res[k];
                    }
                }
            } else {
                acc = wave_xor_sum(acc, kWave);
                if (take_res) {
#pragma unroll
                    for (int k = 0; k < 4; ++k) res[k] = wave_xor_sum(res[k], kWave);
                }
                if (lane == 0) {
                    wsum[wave][0] = acc;
                    if (take_res) { wsum[wave][1] = res[0]; wsum[wave][2] = res[1]; wsum[wave][3] = res[2]; wsum[wave][4] = res[3]; }
                }
                __syncthreads();
                if (threadIdx.x < (take_res ? 5 : 1)) {
                    double s = wsum[0][threadIdx.x];
                    for (int v = 1; v < kWaves; ++v) s += wsum[v][threadIdx.x];
                    if (threadIdx.x == 0) w.p.key[it.g0 + rr] = s;
                    else w.rowres[4 * (int64_t)(it.g0 + rr) + (threadIdx.x - 1)] = s;
                }
                __syncthreads();
            }
        }
    } else {
        const int vw = vec ? 4 : 1;
        const int col = it.col0 + lane * vw;
        const bool in = col < row_len;
        double acc0 = 0.0, acc1 = 0.0, acc2 = 0.0, acc3 = 0.0;
        if (in) {
            for (int rr = wave; rr < it.nr; rr += kWaves) {
                const int64_t e = it.base + (int64_t)rr * row_len + col;
                if (vec) {
                    v4f wb, u, zt;
                    wcand4<R>(w, Rrt, e, al, bl, wb, u, zt);
                    if (w.p.park_mean) st4(w.p.Z + e, wb);
                    acc0 = fma((double)zt.x, (double)zt.x, acc0);
                    acc1 = fma((double)zt.y, (double)zt.y, acc1);
                    acc2 = fma((double)zt.z, (double)zt.z, acc2);
                    acc3 = fma((double)zt.w, (double)zt.w, acc3);
                } else {
                    float wb, u, zt;
                    wcand1<R>(w, Rrt, e, al, bl, wb, u, zt);
                    if (w.p.park_mean) st1(w.p.Z + e, wb);
                    acc0 = fma((double)zt, (double)zt, acc0);
                }
            }
        }
        part[wave][lane * 4 + 0] = acc0;
        part[wave][lane * 4 + 1] = acc1;
        part[wave][lane * 4 + 2] = acc2;
        part[wave][lane * 4 + 3] = acc3;
        __syncthreads();
        if (wave == 0 && in) {
            double* out = w.p.colpart + it.aux + col;
            for (int i = 0; i < vw; ++i) {
                double s = part[0][lane * 4 + i];
                for (int v = 1; v < kWaves; ++v) s += part[v][lane * 4 + i];
                out[i] = s;
            }
        }
    }
}

template <int R, bool RES = false>
__global__ __launch_bounds__(kBlock) void weighted_pass1(const WorkItem* __restrict__ items, WeightedArgs w, int Rrt)
{
    weighted_item<R, RES>(items[blockIdx.x], w, Rrt);
}

// ------------------------------------------------------------------ the weighted projection under a predicted selection

// The candidate of Eq. (9) with everything a final row needs, for 4 (or 1) adjacent elements: the mean, the old
// dual, z~ and the inter-node dual v (what is packed is c = z~ + v).  The arithmetic of wcand4.
template <int R>
__device__ __forceinline__ void wcand4_v(const WeightedArgs& w, int Rrt, int64_t e, float al, float bl,
                                         v4f& wb, v4f& u, v4f& zt, v4f& vd)
{
    const int RR = R > 0 ? R : Rrt;
    v4f s = ld4(w.p.W[0] + e);
#pragma unroll
    for (int r = 1; r < RR; ++r) s = s + ld4(w.p.W[r] + e);
    u = ld4(w.p.Ur + e);
    vd = ld4(w.Vd + e);
    const v4f q = ld4(w.Zg + e) - vd;
    wb = s * w.p.inv_R;
    const v4f t = wb + u;
    const v4f at = t * al;
    const v4f bq = q * bl;
    zt = at + bq;
}

template <int R>
__device__ __forceinline__ void wcand1_v(const WeightedArgs& w, int Rrt, int64_t e, float al, float bl,
                                         float& wb, float& u, float& zt, float& vd)
{
    const int RR = R > 0 ? R : Rrt;
    float s = ld1(w.p.W[0] + e);
#pragma unroll
    for (int r = 1; r < RR; ++r) s = s + ld1(w.p.W[r] + e);
    u = ld1(w.p.Ur + e);
    vd = ld1(w.Vd + e);
    const float q = ld1(w.Zg + e) - vd;
    wb = s * w.p.inv_R;
    const float t = wb + u;
    const float at = t * al;
    const float bq = q * bl;
    zt = at + bq;
}

// One row in the final form of the outcome `kept` (the dual goes to a buffer of its own, so the old dual stays
// readable and either form is final): kept: Z <- z~, U <- U + (Wbar - z~), and c = z~ + v to the packed row `pk`
// unless that is null; pruned: Z <- +0, U <- Wbar + U.  Returns the lane's share of the row's key (the squares of z~
// in the order of weighted_item).  RES: res[0..3] also take the lane's share of the row's residual sums for either
// outcome (see wcand4_res).
template <int R, bool RES = false>
__device__ __forceinline__ double weighted_row_final(const WeightedArgs& w, int Rrt, int64_t base, int row_len, bool vec,
                                                     int j, int step, float al, float bl, bool kept, float* pk,
                                                     double* res = nullptr)
{
    double acc = 0.0;
    const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
    if (vec) {
        const int nchunk = row_len >> 2;
        for (int c = j; c < nchunk; c += step) {
            const int64_t e = base + ((int64_t)c << 2);
            v4f wb, u, zt, vd;
            if (RES) wcand4_res<R>(w, Rrt, e, al, bl, wb, u, zt, vd, res);
            else wcand4_v<R>(w, Rrt, e, al, bl, wb, u, zt, vd);
            st4(w.p.Z + e, kept ? zt : zero4);
            st4(w.p.U + e, kept ? u + (wb - zt) : wb + u);
            if (pk) st4u(pk + 4 * c, zt + vd);
            if (w.p.Wbar) st4(w.p.Wbar + e, wb);
            acc = sq4(acc, zt);
        }
    } else {
        for (int c = j; c < row_len; c += step) {
            float wb, u, zt, vd;
            if (RES) wcand1_res<R>(w, Rrt, base + c, al, bl, wb, u, zt, vd, res);
            else wcand1_v<R>(w, Rrt, base + c, al, bl, wb, u, zt, vd);
            st1(w.p.Z + base + c, kept ? zt : 0.f);
            st1(w.p.U + base + c, kept ? u + (wb - zt) : wb + u);
            if (pk) pk[c] = zt + vd;
            if (w.p.Wbar) st1(w.p.Wbar + base + c, wb);
            acc = fma((double)zt, (double)zt, acc);
        }
    }
    return acc;
}

// What the weighted pass 1 needs under a prediction (see HintArgs in kernels_project.hpp for the records).
struct WeightedHint {
    const int32_t* sel_prev;
    float* packed;      // null: no compaction
    int32_t* work;      // the work list's counter is cleared here
    const DevLayer* layers;
};

// Row items of FILTER and unconstrained layers under a predicted selection, dual out of place: every row is written
// in the final form of its predicted outcome and, if predicted kept, packed at its predicted rank (ranks outside
// [0, k) are left for the repair pass).  The keys are taken with the lane mapping of weighted_item; its sums run
// two chunks at a time where this loop takes one, in the same order of additions.  RES: as in weighted_item, the
// residual sums of either outcome of every row go to rowres (the selection picks by the real outcome, so a wrong
// prediction costs them nothing).
template <int R, bool RES>
__device__ __forceinline__ void weighted_rows_hinted(const WorkItem& it, const WeightedArgs& w, int Rrt,
                                                     const WeightedHint& h)
{
    __shared__ double wsum[kWaves][5];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = it.row_len;
    const bool vec = item_vec(it);
    const float al = w.coef[2 * it.layer], bl = w.coef[2 * it.layer + 1];
    const bool unconstrained = item_mode(it) == HSADMM_MODE_NONE;
    const bool wide = it.lpr > kWave;
    const int lpr = wide ? kBlock : it.lpr;
    const int rows_at_once = kBlock / lpr;
    const int sub = threadIdx.x / lpr;
    const int j = threadIdx.x - sub * lpr;
    const int rounds = (it.nr + rows_at_once - 1) / rows_at_once;
    float* const pk_layer = h.packed ? h.packed + it.packed_off : nullptr;
    for (int rd = 0; rd < rounds; ++rd) {
        const int rr = rd * rows_at_once + sub;
        const bool active = rr < it.nr;
        double acc = 0.0;
        double res[4] = {0.0, 0.0, 0.0, 0.0};
        if (active) {
            const int hp = unconstrained ? it.row0 + rr : h.sel_prev[it.g0 + rr];
            const bool kept = hp >= 0;
            float* pk = (pk_layer && kept && hp < it.k) ? pk_layer + (int64_t)hp * row_len : nullptr;
            acc = weighted_row_final<R, RES>(w, Rrt, it.base + (int64_t)rr * row_len, row_len, vec, j, lpr, al, bl, kept,
                                             pk, res);
        }
        if (!wide) {
            acc = wave_xor_sum(acc, lpr);
            if (active && j == 0) w.p.key[it.g0 + rr] = acc;
            if (RES) {
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    res[k] = wave_xor_sum(res[k], lpr);
                    if (active && j == 0) w.rowres[4 * (int64_t)(it.g0 + rr) + k] = res[k];
                }
            }
        } else {
            acc = wave_xor_sum(acc, kWave);
            if (RES) {
#pragma unroll
                for (int k = 0; k < 4; ++k) res[k] = wave_xor_sum(res[k], kWave);
            }
            if (lane == 0) {
                wsum[wave][0] = acc;
                if (RES) { wsum[wave][1] = res[0]; wsum[wave][2] = res[1]; wsum[wave][3] = res[2]; wsum[wave][4] = res[3]; }
            }
            __syncthreads();
            if (threadIdx.x < (RES ? 5 : 1)) {
                double s = wsum[0][threadIdx.x];
                for (int v = 1; v < kWaves; ++v) s += wsum[v][threadIdx.x];
                if (threadIdx.x == 0) w.p.key[it.g0 + rr] = s;
                else w.rowres[4 * (int64_t)(it.g0 + rr) + (threadIdx.x - 1)] = s;
            }
            __syncthreads();
        }
    }
}

// TILES: CHANNEL and BOTH layers take the prediction as well (the weighted forms of project_tile_hinted and
// project_rows_both_hinted; an instantiation of its own for plans with such layers, so that the other plans' kernel
// keeps its registers); else they only sum here (and park) and are written after the selection.
template <int R, bool RES = false, bool TILES = false>
__global__ __launch_bounds__(kBlock) void weighted_pass1_hinted(const WorkItem* __restrict__ items, WeightedArgs w,
                                                                int Rrt, WeightedHint h)
{
    const WorkItem it = items[blockIdx.x];
    const int mode = item_mode(it);
    if (blockIdx.x == 0 && threadIdx.x == 0) h.work[0] = 0;      // (the selection runs after this whole launch)
    if (mode == HSADMM_MODE_FILTER || mode == HSADMM_MODE_NONE) {
        weighted_rows_hinted<R, RES>(it, w, Rrt, h);
    } else if constexpr (TILES) {                                // (CHANNEL and BOTH layers take no residual sums here)
        const HintArgs hh{h.sel_prev, h.packed, 0, h.work, h.layers};
        if (mode == HSADMM_MODE_CHANNEL) project_tile_hinted<R, true>(it, w.p, Rrt, hh);
        else project_rows_both_hinted<R, true>(it, w.p, Rrt, hh);
    } else {
        weighted_item<R, false>(it, w, Rrt);
    }
}

// The repair pass of the weighted projection under a prediction: a fixed grid shares the row items the selection has
// listed.  A FILTER row whose prediction was wrong is formed again from the inputs in the form of its real outcome; a
// kept row whose rank has moved is copied to its new place in the packed buffer as c = Z + v.  A listed item of a
// CHANNEL or BOTH layer belongs to a layer whose selection differs from its record: its rows are formed again under
// the mask just selected (the frozen-mask pass in its weighted form; po.packed null: no compaction).
template <int R>
__global__ __launch_bounds__(kBlock) void weighted_hinted_repair(const WorkItem* __restrict__ row_items, WeightedArgs w,
                                                                 int Rrt, WeightedHint h, const int32_t* __restrict__ pos,
                                                                 const uint8_t* __restrict__ mask, PackOut po)
{
    const int n = h.work[0];
    for (int i = blockIdx.x; i < n; i += gridDim.x) {
        const WorkItem it = row_items[h.work[kWorkHeader + i]];
        if (mode_has_channels(item_mode(it))) {
            if (po.packed) frozen_item<R, true, true>(it, w.p, Rrt, mask, po);
            else frozen_item<R, false, true>(it, w.p, Rrt, mask, po);
            continue;
        }
        if (item_mode(it) != HSADMM_MODE_FILTER) continue;
        const int row_len = it.row_len;
        const bool vec = item_vec(it);
        const float al = w.coef[2 * it.layer], bl = w.coef[2 * it.layer + 1];
        const int lpr = it.lpr <= kWave ? it.lpr : kBlock;
        const int rows_at_once = kBlock / lpr;
        const int sub = threadIdx.x / lpr;
        const int j = threadIdx.x - sub * lpr;
        float* const pk_layer = h.packed ? h.packed + it.packed_off : nullptr;
        for (int rr = sub; rr < it.nr; rr += rows_at_once) {
            const int hp = h.sel_prev[it.g0 + rr];
            const int pn = pos[it.g0 + rr];
            const bool pred_kept = hp >= 0, kept = pn >= 0;
            const int64_t base = it.base + (int64_t)rr * row_len;
            float* pk = (pk_layer && kept) ? pk_layer + (int64_t)pn * row_len : nullptr;
            if (pred_kept != kept) {
                (void)weighted_row_final<R>(w, Rrt, base, row_len, vec, j, lpr, al, bl, kept, pk);
            } else if (pk && pn != hp) {
                if (vec) for (int c = j; c < (row_len >> 2); c += lpr) st4u(pk + 4 * c, ld4(w.p.Z + base + 4 * c) + ld4(w.Vd + base + 4 * c));
                else for (int c = j; c < row_len; c += lpr) pk[c] = ld1(w.p.Z + base + c) + ld1(w.Vd + base + c);
            }
        }
    }
}

// FILTER layers once the mask is known (row items): Z holds t = Wbar + U and U the kept form.
//   kept filter:   Z <- z~ = fl(fl(a t) + fl(b (Zg - Vd)))   (the arithmetic of wcand4, from the stashed t)
//   pruned filter: U <- t (= U + (Wbar - 0) bit for bit), Z <- +0
// PACK: a kept row also goes to the packed buffer as c = z~ + Vd (the pre-transmission buffer z_i + v_i of Section
// 4.4.1, which hsadmm_compact_sum would form from Z and Vd), at the row's rank under the selection's index mappings.
template <bool PACK>
__device__ __forceinline__ void weighted_fixup_rows(const WorkItem& it, const uint8_t* mask, float* U, float* Z,
                                                    const float* Zg, const float* Vd, const float* coef,
                                                    const PackOut& po)
{
    const int row_len = it.row_len;
    const bool vec = item_vec(it);
    const float al = coef[2 * it.layer], bl = coef[2 * it.layer + 1];
    const int lpr = it.lpr <= kWave ? it.lpr : kBlock;
    const int rows_at_once = kBlock / lpr;
    const int sub = threadIdx.x / lpr;
    const int j = threadIdx.x - sub * lpr;
    const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
    float* out = nullptr;
    if (PACK) {
        if (it.row0 == 0) copy_out_layer(it.layer, po.cnt, po.kept_idx, po.n_layers, po.layer_off, po.co);
        out = po.packed + po.layer_off[it.layer];
    }
    for (int rr = sub; rr < it.nr; rr += rows_at_once) {
        const bool keep = mask[it.g0 + rr] != 0;
        const int64_t base = it.base + (int64_t)rr * row_len;
        float* d = nullptr;
        if (PACK && keep) d = out + (int64_t)po.pos[it.g0 + rr] * row_len;
        if (vec) {
            const int nchunk = row_len >> 2;
            for (int c = j; c < nchunk; c += lpr) {
                const int64_t e = base + ((int64_t)c << 2);
                const v4f t = ld4(Z + e);
                if (keep) {
                    const v4f vd = ld4(Vd + e);
                    const v4f q = ld4(Zg + e) - vd;
                    const v4f at = t * al;
                    const v4f bq = q * bl;
                    const v4f z = at + bq;
                    st4(Z + e, z);
                    if (PACK) st4u(d + 4 * c, z + vd);
                } else {
                    st4(U + e, t);
                    st4(Z + e, zero4);
                }
            }
        } else {
            for (int c = j; c < row_len; c += lpr) {
                const int64_t e = base + c;
                const float t = ld1(Z + e);
                if (keep) {
                    const float vd = ld1(Vd + e);
                    const float q = ld1(Zg + e) - vd;
                    const float at = t * al;
                    const float bq = q * bl;
                    const float z = at + bq;
                    st1(Z + e, z);
                    if (PACK) d[c] = z + vd;
                } else {
                    st1(U + e, t);
                    st1(Z + e, 0.f);
                }
            }
        }
    }
}

__global__ __launch_bounds__(kBlock) void weighted_fixup(const WorkItem* __restrict__ items,
                                                         const uint8_t* __restrict__ mask,
                                                         float* __restrict__ U, float* __restrict__ Z,
                                                         const float* __restrict__ Zg, const float* __restrict__ Vd,
                                                         const float* __restrict__ coef)
{
    weighted_fixup_rows<false>(items[blockIdx.x], mask, U, Z, Zg, Vd, coef, PackOut{});
}

// Eq. (13): v <- v + (z_i - z) over every layer.  A row item is one contiguous span of the arena.
__global__ __launch_bounds__(kBlock) void dual_inter_kernel(const WorkItem* __restrict__ items,
                                                            const float* __restrict__ Zi,
                                                            const float* __restrict__ Zg, float* __restrict__ Vd)
{
    const WorkItem it = items[blockIdx.x];
    const int64_t len = (int64_t)it.nr * it.row_len;
    if (item_vec(it)) {
        for (int64_t c = threadIdx.x; c < (len >> 2); c += kBlock) {
            const int64_t e = it.base + (c << 2);
            const v4f d = ld4(Zi + e) - ld4(Zg + e);
            st4(Vd + e, ld4(Vd + e) + d);
        }
    } else {
        for (int64_t c = threadIdx.x; c < len; c += kBlock) {
            const int64_t e = it.base + c;
            const float d = Zi[e] - Zg[e];
            Vd[e] = Vd[e] + d;
        }
    }
}

// X <- fl(X * factor[layer]) over every layer: a scaled dual follows its layer's penalty (u = y / rho is multiplied
// by rho_old / rho_new when the adaptive tuning of Section 3.4 changes rho).  Items of a layer whose factor is 1 do
// nothing, so an iteration that changes few penalties moves few bytes.
__global__ __launch_bounds__(kBlock) void scale_layers_kernel(const WorkItem* __restrict__ items,
                                                              const float* __restrict__ factor, float* __restrict__ X)
{
    const WorkItem it = items[blockIdx.x];
    const float f = factor[it.layer];
    if (f == 1.0f) return;
    const int64_t len = (int64_t)it.nr * it.row_len;
    if (item_vec(it)) {
        for (int64_t c = threadIdx.x; c < (len >> 2); c += kBlock) {
            const int64_t e = it.base + (c << 2);
            st4(X + e, ld4(X + e) * f);
        }
    } else {
        for (int64_t c = threadIdx.x; c < len; c += kBlock) X[it.base + c] = X[it.base + c] * f;
    }
}

// Eq. (11): global consensus z = (1/M) sum_i (z_i + v_i) over M equally long buffers (the nodes' compact
// pre-transmission buffers): fp32 sum in node order, times fl32(1/M).  Flat grid-stride stream.
struct AverageArgs {
    const float* b[HSADMM_MAX_MASKS];
};

__global__ __launch_bounds__(kBlock) void average_kernel(AverageArgs a, int M, float inv_M, int64_t n,
                                                         float* out /* may be one of the inputs */)
{
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    const int64_t quads = n >> 2;
    for (int64_t q = (int64_t)blockIdx.x * kBlock + threadIdx.x; q < quads; q += stride) {
        const int64_t e = q << 2;
        v4f s = ld4(a.b[0] + e);
        for (int i = 1; i < M; ++i) s = s + ld4(a.b[i] + e);
        st4(out + e, s * inv_M);
    }
    // the last n % 4 elements
    const int64_t e = (quads << 2) + (int64_t)blockIdx.x * kBlock + threadIdx.x;
    if (e < n) {
        float s = a.b[0][e];
        for (int i = 1; i < M; ++i) s = s + a.b[i][e];
        out[e] = s * inv_M;
    }
}

}  // namespace
#endif
