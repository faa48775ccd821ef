// hsadmm_project_frozen / hsadmm_project_weighted_frozen (a given mask applied in one pass; the same kernel is the
// final pass of CHANNEL and BOTH layers in the dynamic projections), hsadmm_mask_or and hsadmm_mask_drift.
// Part of the single translation unit built from hsadmm.hip (included there, in order).
#ifndef KERNELS_FROZEN_HPP
#define KERNELS_FROZEN_HPP
#include "hsadmm_device.hpp"

namespace {

// ------------------------------------------------------------------ project under a frozen mask

// R = kMeanInZ: the mean of the replicas is not formed here but read from Z, where pass 1 parked it.
constexpr int kMeanInZ = -1;

// Final values of 4 adjacent elements under a known mask (Algorithm 1 Phase 3, retraining branch:
// z = z~ (.) m): kept element Z = V, U += Wbar - V; masked-out element Z = +0, U = U + Wbar (= V).
// PACK: d, when not null, is where the 4 elements go in the packed buffer (rows packed whole).
// WEIGHTED: the candidate is z~ = fl(fl(a t) + fl(b (Zg - Vd))), t = Wbar + U (Eq. (9)), and what is packed is
// c = z + Vd (Section 4.4.1); else the candidate is t and what is packed is z.  The value packed is returned.
// RES: Z holds the previous z_i on entry; acc[0] += sum_j (W_j - z)^2 and acc[1] += (z - z_prev)^2 over the
// 4 elements, in fp64 (the intra-node primal and dual residuals of Section 3.4).  With a compile-time R the
// replicas' values stay in registers for this; with a run-time R they are read a second time.
template <int R, bool PACK = false, bool WEIGHTED = false, bool RES = false>
__device__ __forceinline__ v4f frozen4(const ProjectArgs& a, int Rrt, int64_t e, bool k0, bool k1, bool k2, bool k3,
                                       float* d = nullptr, float al = 1.f, float bl = 0.f, double* acc = nullptr)
{
    static_assert(!RES || R != kMeanInZ, "the residual norms need the replicas");
    constexpr int kHeld = (RES && R > 0) ? R : 1;
    v4f w[kHeld];
    v4f wb;
    if (R == kMeanInZ) {
        wb = ld4(a.Z + e);
    } else {
        const int RR = R > 0 ? R : Rrt;
        v4f s = ld4(a.W[0] + e);
        if (RES && R > 0) w[0] = s;
#pragma unroll
        for (int r = 1; r < RR; ++r) {
            const v4f x = ld4(a.W[r] + e);
            if (RES && R > 0) w[r] = x;
            s = s + x;
        }
        wb = s * a.inv_R;
    }
    v4f zprev = {0.f, 0.f, 0.f, 0.f};
    if (RES) zprev = ld4(a.Z + e);
    const v4f u = ld4(a.Ur + e);
    v4f v = wb + u;
    v4f vd = {0.f, 0.f, 0.f, 0.f};
    if (WEIGHTED) {
        vd = ld4(a.Vd + e);
        const v4f q = ld4(a.Zg + e) - vd;
        const v4f at = v * al;
        const v4f bq = q * bl;
        v = at + bq;
    }
    v4f z;
    z.x = k0 ? v.x : 0.f; z.y = k1 ? v.y : 0.f; z.z = k2 ? v.z : 0.f; z.w = k3 ? v.w : 0.f;
    st4(a.Z + e, z);
    st4(a.U + e, u + (wb - z));
    if (a.Wbar) st4(a.Wbar + e, wb);
    const v4f c = WEIGHTED ? z + vd : z;
    if (PACK && d) st4u(d, c);
    if (RES) {
        const int RR = R > 0 ? R : Rrt;
        acc[1] = sqd4(acc[1], z, zprev);
#pragma unroll
        for (int r = 0; r < RR; ++r) acc[0] = sqd4(acc[0], R > 0 ? w[r] : ld4(a.W[r] + e), z);
    }
    return c;
}

// two chunks of one row (same keep flag) with all loads issued before any store
template <int R, bool PACK = false, bool WEIGHTED = false, bool RES = false>
__device__ __forceinline__ void frozen4x2(const ProjectArgs& a, int Rrt, int64_t e0, int64_t e1, bool keep,
                                          float* d0 = nullptr, float* d1 = nullptr, float al = 1.f, float bl = 0.f,
                                          double* acc = nullptr)
{
    constexpr int kHeld = (RES && R > 0) ? R : 1;
    v4f wa[kHeld], wc[kHeld];
    v4f wb0, wb1;
    if (R == kMeanInZ) {
        wb0 = ld4(a.Z + e0);
        wb1 = ld4(a.Z + e1);
    } else {
        const int RR = R > 0 ? R : Rrt;
        v4f s0 = ld4(a.W[0] + e0), s1 = ld4(a.W[0] + e1);
        if (RES && R > 0) { wa[0] = s0; wc[0] = s1; }
#pragma unroll
        for (int r = 1; r < RR; ++r) {
            const v4f w0 = ld4(a.W[r] + e0), w1 = ld4(a.W[r] + e1);
            if (RES && R > 0) { wa[r] = w0; wc[r] = w1; }
            s0 = s0 + w0;
            s1 = s1 + w1;
        }
        wb0 = s0 * a.inv_R;
        wb1 = s1 * a.inv_R;
    }
    const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
    v4f zp0 = zero4, zp1 = zero4;
    if (RES) { zp0 = ld4(a.Z + e0); zp1 = ld4(a.Z + e1); }
    const v4f u0 = ld4(a.Ur + e0), u1 = ld4(a.Ur + e1);
    v4f v0 = wb0 + u0, v1 = wb1 + u1;
    v4f vd0 = zero4, vd1 = zero4;
    if (WEIGHTED && keep) {         // a pruned row needs neither z nor v
        vd0 = ld4(a.Vd + e0);
        vd1 = ld4(a.Vd + e1);
        const v4f q0 = ld4(a.Zg + e0) - vd0, q1 = ld4(a.Zg + e1) - vd1;
        const v4f at0 = v0 * al, at1 = v1 * al;
        const v4f bq0 = q0 * bl, bq1 = q1 * bl;
        v0 = at0 + bq0;
        v1 = at1 + bq1;
    }
    const v4f z0 = keep ? v0 : zero4, z1 = keep ? v1 : zero4;
    st4(a.Z + e0, z0);
    st4(a.Z + e1, z1);
    st4(a.U + e0, u0 + (wb0 - z0));
    st4(a.U + e1, u1 + (wb1 - z1));
    if (a.Wbar) { st4(a.Wbar + e0, wb0); st4(a.Wbar + e1, wb1); }
    if (PACK && d0) { st4u(d0, WEIGHTED ? z0 + vd0 : z0); st4u(d1, WEIGHTED ? z1 + vd1 : z1); }
    if (RES) {
        const int RR = R > 0 ? R : Rrt;
        acc[1] = sqd4(acc[1], z0, zp0);
        acc[1] = sqd4(acc[1], z1, zp1);
#pragma unroll
        for (int r = 0; r < RR; ++r) {
            acc[0] = sqd4(acc[0], R > 0 ? wa[r] : ld4(a.W[r] + e0), z0);
            acc[0] = sqd4(acc[0], R > 0 ? wc[r] : ld4(a.W[r] + e1), z1);
        }
    }
}

template <int R, bool PACK = false, bool WEIGHTED = false, bool RES = false>
__device__ __forceinline__ float frozen1(const ProjectArgs& a, int Rrt, int64_t e, bool keep, float* d = nullptr,
                                         float al = 1.f, float bl = 0.f, double* acc = nullptr)
{
    float zprev = 0.f;
    if (RES) zprev = ld1(a.Z + e);
    float wb;
    if (R == kMeanInZ) {
        wb = ld1(a.Z + e);
    } else {
        const int RR = R > 0 ? R : Rrt;
        float s = ld1(a.W[0] + e);
#pragma unroll
        for (int r = 1; r < RR; ++r) s = s + ld1(a.W[r] + e);
        wb = s * a.inv_R;
    }
    const float u = ld1(a.Ur + e);
    float v = wb + u;
    float vd = 0.f;
    if (WEIGHTED) {
        vd = ld1(a.Vd + e);
        const float q = ld1(a.Zg + e) - vd;
        const float at = v * al;
        const float bq = q * bl;
        v = at + bq;
    }
    const float z = keep ? v : 0.f;
    st1(a.Z + e, z);
    st1(a.U + e, u + (wb - z));
    if (a.Wbar) st1(a.Wbar + e, wb);
    const float c = WEIGHTED ? z + vd : z;
    if (PACK && d) *d = c;
    if (RES) {
        const int RR = R > 0 ? R : Rrt;
        acc[1] = sqd(acc[1], z, zprev);
        for (int r = 0; r < RR; ++r) acc[0] = sqd(acc[0], ld1(a.W[r] + e), z);
    }
    return c;
}

// pc[i] = the packed column of column col + i, or -1 if its channel is not kept (rank: the ranks of the layer's
// channels among the kept ones, -1 for a pruned channel), for 4 adjacent columns.
__device__ __forceinline__ void quad_packed_cols(const int32_t* __restrict__ rank, const DivKhw& div, int col,
                                                 int pc[4])
{
    if (div.khw == 1) {
        int4 r;
        __builtin_memcpy(&r, rank + col, 16);
        pc[0] = r.x; pc[1] = r.y; pc[2] = r.z; pc[3] = r.w;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int ch = div(col + i);
            const int r = rank[ch];
            pc[i] = r < 0 ? -1 : r * div.khw + (col + i - ch * div.khw);
        }
    }
}

// Row items of every mode (the compact / expand item table): no keys, no second pass, every byte of the
// replicas (or of the parked mean) and of U is read once and Z and U are written once, streaming along the rows.  FILTER / NONE rows
// share one keep flag; in CHANNEL rows and in the kept filters' rows of a BOTH layer every column takes the
// flag of its channel.
// PACK: what the mask keeps also goes to the packed buffer as it is formed, under the index mappings of this
// mask (po): a kept FILTER row or a row of a NONE layer whole, at its rank; of a CHANNEL row, or a kept filter's
// row of a BOTH layer, the columns of kept channels, each at its packed column.
// RES: acc[0], acc[1] take this thread's share of the item's two intra-node residual sums (see frozen4).
template <int R, bool PACK, bool WEIGHTED = false, bool RES = false>
__device__ __forceinline__ void frozen_item(const WorkItem& it, const ProjectArgs& a, int Rrt,
                                            const uint8_t* __restrict__ mask, const PackOut& po,
                                            double* acc = nullptr)
{
    const int mode = item_mode(it);
    const float al = WEIGHTED ? a.coef[2 * it.layer] : 1.f, bl = WEIGHTED ? a.coef[2 * it.layer + 1] : 0.f;
    const int row_len = it.row_len;
    const bool vec = item_vec(it);
    const int lpr = it.lpr <= kWave ? it.lpr : kBlock;
    const int rows_at_once = kBlock / lpr;
    const int sub = threadIdx.x / lpr;
    const int j = threadIdx.x - sub * lpr;
    const bool columns = mode_has_channels(mode);
    // channel bytes of the layer (CHANNEL row item: g0 is the layer's first group)
    const uint8_t* mc = mask + (mode == HSADMM_MODE_BOTH ? it.aux : (int64_t)it.g0);
    const DivKhw div(it.khw);
    float* out = nullptr;
    int packed_row_len = 0;                 // rows that keep a subset of their columns: kept channels * khw
    const int32_t* rank = nullptr;          // ... and the ranks of the layer's channels
    if (PACK) {
        if (it.row0 == 0) copy_out_layer(it.layer, po.cnt, po.kept_idx, po.n_layers, po.layer_off, po.co);
        out = po.packed + po.layer_off[it.layer];
        if (columns) {
            const int kc = mode == HSADMM_MODE_BOTH ? po.cnt[2 * po.n_layers + it.layer] : po.cnt[it.layer];
            packed_row_len = kc * it.khw;
            rank = po.pos + (mode == HSADMM_MODE_BOTH ? it.aux : (int64_t)it.g0);
        }
    }
    for (int rr = sub; rr < it.nr; rr += rows_at_once) {
        const bool keep = mode == HSADMM_MODE_NONE || mode == HSADMM_MODE_CHANNEL || mask[it.g0 + rr] != 0;
        const int64_t base = it.base + (int64_t)rr * row_len;
        if (columns && keep) {
            float* drow = nullptr;          // this row in the packed buffer
            if (PACK) {
                const int p = mode == HSADMM_MODE_CHANNEL ? it.row0 + rr : po.pos[it.g0 + rr];
                if (p >= 0) drow = out + (int64_t)p * packed_row_len;
            }
            if (vec) {
                const int nchunk = row_len >> 2;
                for (int c = j; c < nchunk; c += lpr) {
                    const int col = c << 2;
                    bool pr[4];
                    quad_pruned(mc, div, col, pr);
                    const v4f z = frozen4<R, false, WEIGHTED, RES>(a, Rrt, base + col, !pr[0], !pr[1], !pr[2], !pr[3], nullptr, al, bl, acc);
                    if (PACK && drow) {
                        int pc[4];
                        quad_packed_cols(rank, div, col, pc);
                        if (pc[0] >= 0) drow[pc[0]] = z.x;
                        if (pc[1] >= 0) drow[pc[1]] = z.y;
                        if (pc[2] >= 0) drow[pc[2]] = z.z;
                        if (pc[3] >= 0) drow[pc[3]] = z.w;
                    }
                }
            } else {
                for (int c = j; c < row_len; c += lpr) {
                    const int ch = div(c);
                    const float z = frozen1<R, false, WEIGHTED, RES>(a, Rrt, base + c, mc[ch] != 0, nullptr, al, bl, acc);
                    if (PACK && drow) {
                        const int r = rank[ch];
                        if (r >= 0) drow[r * it.khw + (c - ch * it.khw)] = z;
                    }
                }
            }
            continue;
        }
        // a kept row of a FILTER or NONE layer is packed whole, at its rank (NONE: its own index)
        float* d = nullptr;
        if (PACK && !columns && keep) {
            const int p = mode == HSADMM_MODE_NONE ? it.row0 + rr : po.pos[it.g0 + rr];
            if (p >= 0) d = out + (int64_t)p * row_len;     // (mappings of another mask: the row is left out)
        }
        if (vec) {
            const int nchunk = row_len >> 2;
            int c = j;
            for (; c + lpr < nchunk; c += 2 * lpr)
                frozen4x2<R, PACK, WEIGHTED, RES>(a, Rrt, base + ((int64_t)c << 2), base + ((int64_t)(c + lpr) << 2), keep,
                                                  d ? d + 4 * c : nullptr, d ? d + 4 * (c + lpr) : nullptr, al, bl, acc);
            if (c < nchunk)
                frozen4<R, PACK, WEIGHTED, RES>(a, Rrt, base + ((int64_t)c << 2), keep, keep, keep, keep,
                                                d ? d + 4 * c : nullptr, al, bl, acc);
        } else {
            for (int c = j; c < row_len; c += lpr)
                frozen1<R, PACK, WEIGHTED, RES>(a, Rrt, base + c, keep, d ? d + c : nullptr, al, bl, acc);
        }
    }
}

// RES: the item's two intra-node residual sums also go to a.respart[4 * item + 0, 1].
template <int R, bool PACK = false, bool WEIGHTED = false, bool RES = false>
__global__ __launch_bounds__(kBlock) void project_frozen(const WorkItem* __restrict__ items, ProjectArgs a, int Rrt,
                                                         const uint8_t* __restrict__ mask, PackOut po)
{
    if constexpr (RES) {
        double acc[2] = {0.0, 0.0};
        frozen_item<R, PACK, WEIGHTED, true>(items[blockIdx.x], a, Rrt, mask, po, acc);
        block_sum_pair(acc[0], acc[1], a.respart + (int64_t)blockIdx.x * 4);
    } else {
        frozen_item<R, PACK, WEIGHTED, false>(items[blockIdx.x], a, Rrt, mask, po);
    }
}

// Eq. (14): out = OR of M masks, 0 / 1 bytes.
struct MaskOrArgs {
    const uint8_t* m[HSADMM_MAX_MASKS];
};

__global__ __launch_bounds__(kBlock) void mask_or_kernel(MaskOrArgs a, int M, int64_t n,
                                                         uint8_t* out /* may be one of the inputs */)
{
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t g = (int64_t)blockIdx.x * kBlock + threadIdx.x; g < n; g += stride) {
        unsigned int any = 0;
        for (int i = 0; i < M; ++i) any |= a.m[i][g];
        out[g] = any != 0 ? 1 : 0;
    }
}

// Section 4.5 (mask freezing once the pattern is stable): per layer, the number of groups whose kept flag differs
// between two masks.  One workgroup per layer; an unconstrained layer reports 0.
__global__ __launch_bounds__(kBlock) void mask_drift_kernel(const DevLayer* __restrict__ layers,
                                                            const uint8_t* __restrict__ a,
                                                            const uint8_t* __restrict__ b,
                                                            int32_t* __restrict__ drift)
{
    __shared__ int wsum[kWaves];
    const DevLayer L = layers[blockIdx.x];
    int d = 0;
    if (L.mode != HSADMM_MODE_NONE)
        for (int g = threadIdx.x; g < L.G; g += kBlock)
            d += ((a[L.group_base + g] != 0) != (b[L.group_base + g] != 0)) ? 1 : 0;
    d = wave_sum_i32(d);
    if ((threadIdx.x & (kWave - 1)) == 0) wsum[threadIdx.x / kWave] = d;
    __syncthreads();
    if (threadIdx.x == 0) {
        int t = 0;
        for (int w = 0; w < kWaves; ++w) t += wsum[w];
        drift[blockIdx.x] = t;
    }
}

}  // namespace
#endif
