// hsadmm_project: streaming pass 1 (mean, candidate, fp64 group sums, speculative outputs) and the fix-up of pruned groups.
// Part of the single translation unit built from hsadmm.hip (included there, in order).
#ifndef KERNELS_PROJECT_HPP
#define KERNELS_PROJECT_HPP
#include "hsadmm_device.hpp"

namespace {

// ------------------------------------------------------------------ project, pass 1

__device__ __forceinline__ double sq4(double acc, const v4f& v)
{
    acc = fma((double)v.x, (double)v.x, acc);
    acc = fma((double)v.y, (double)v.y, acc);
    acc = fma((double)v.z, (double)v.z, acc);
    acc = fma((double)v.w, (double)v.w, acc);
    return acc;
}

// Wbar, V and the dual value that is final if the group is kept, for 4 (or 1) adjacent elements.
// R > 0: replica count known at compile time (loop unrolled, pointers stay in scalar registers);
// R == 0: any replica count, taken from Rrt.
template <int R>
struct Cand {
    // two independent 4-element chunks at once (twice the loads in flight)
    static __device__ __forceinline__ double two(const ProjectArgs& a, int Rrt, int64_t e0, int64_t e1, double acc)
    {
        const int RR = R > 0 ? R : Rrt;
        v4f s0 = ld4(a.W[0] + e0), s1 = ld4(a.W[0] + e1);
#pragma unroll
        for (int r = 1; r < RR; ++r) {
            const v4f w0 = ld4(a.W[r] + e0), w1 = ld4(a.W[r] + e1);
            s0 = s0 + w0;
            s1 = s1 + w1;
        }
        const v4f u0 = ld4(a.Ur + e0), u1 = ld4(a.Ur + e1);
        const v4f wb0 = s0 * a.inv_R, wb1 = s1 * a.inv_R;
        const v4f v0 = wb0 + u0, v1 = wb1 + u1;
        const v4f d0 = wb0 - v0, d1 = wb1 - v1;
        st4(a.Z + e0, v0);
        st4(a.Z + e1, v1);
        st4(a.U + e0, u0 + d0);
        st4(a.U + e1, u1 + d1);
        if (a.Wbar) { st4(a.Wbar + e0, wb0); st4(a.Wbar + e1, wb1); }
        acc = sq4(acc, v0);
        return sq4(acc, v1);
    }
    static __device__ __forceinline__ v4f one(const ProjectArgs& a, int Rrt, int64_t e)
    {
        const int RR = R > 0 ? R : Rrt;
        v4f s = ld4(a.W[0] + e);
#pragma unroll
        for (int r = 1; r < RR; ++r) s = s + ld4(a.W[r] + e);
        const v4f u = ld4(a.Ur + e);
        const v4f wb = s * a.inv_R;
        const v4f v = wb + u;
        const v4f d = wb - v;
        st4(a.Z + e, v);
        st4(a.U + e, u + d);
        if (a.Wbar) st4(a.Wbar + e, wb);
        return v;
    }
    // HINTED forms: a previous selection predicts the row's fate (`kept`), and the row is written in the form that
    // fate makes final.  Predicted kept: Z <- V, U <- U + (Wbar - V), as always.  Predicted pruned: U <- V, and
    // Z <- the dual of a kept group when `stash` (the dual is updated in place and its old value is lost here: either
    // outcome can then still be finished without the replicas), else Z <- +0 (the old dual stays readable in
    // another buffer, so a wrong prediction is repaired from the inputs).  `pk`, unless null, is the row's place
    // in the packed buffer.
    static __device__ __forceinline__ void put_h(const ProjectArgs& a, int64_t e, const v4f& v, const v4f& dual_kept,
                                                 bool kept, bool stash)
    {
        const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
        const v4f other = stash ? dual_kept : zero4;
        st4(a.Z + e, kept ? v : other);
        st4(a.U + e, kept ? dual_kept : v);
    }
    static __device__ __forceinline__ double two_h(const ProjectArgs& a, int Rrt, int64_t base, int o0, int o1,
                                                   bool kept, bool stash, float* pk, double acc)
    {
        const int RR = R > 0 ? R : Rrt;
        const int64_t e0 = base + o0, e1 = base + o1;
        v4f s0 = ld4(a.W[0] + e0), s1 = ld4(a.W[0] + e1);
#pragma unroll
        for (int r = 1; r < RR; ++r) {
            const v4f w0 = ld4(a.W[r] + e0), w1 = ld4(a.W[r] + e1);
            s0 = s0 + w0;
            s1 = s1 + w1;
        }
        const v4f u0 = ld4(a.Ur + e0), u1 = ld4(a.Ur + e1);
        const v4f wb0 = s0 * a.inv_R, wb1 = s1 * a.inv_R;
        const v4f v0 = wb0 + u0, v1 = wb1 + u1;
        const v4f d0 = wb0 - v0, d1 = wb1 - v1;
        put_h(a, e0, v0, u0 + d0, kept, stash);
        put_h(a, e1, v1, u1 + d1, kept, stash);
        if (pk) { st4u(pk + o0, v0); st4u(pk + o1, v1); }
        if (a.Wbar) { st4(a.Wbar + e0, wb0); st4(a.Wbar + e1, wb1); }
        acc = sq4(acc, v0);
        return sq4(acc, v1);
    }
    static __device__ __forceinline__ v4f one_h(const ProjectArgs& a, int Rrt, int64_t base, int o, bool kept,
                                                bool stash, float* pk)
    {
        const int RR = R > 0 ? R : Rrt;
        const int64_t e = base + o;
        v4f s = ld4(a.W[0] + e);
#pragma unroll
        for (int r = 1; r < RR; ++r) s = s + ld4(a.W[r] + e);
        const v4f u = ld4(a.Ur + e);
        const v4f wb = s * a.inv_R;
        const v4f v = wb + u;
        const v4f d = wb - v;
        put_h(a, e, v, u + d, kept, stash);
        if (pk) st4u(pk + o, v);
        if (a.Wbar) st4(a.Wbar + e, wb);
        return v;
    }
    static __device__ __forceinline__ float scalar_h(const ProjectArgs& a, int Rrt, int64_t base, int o, bool kept,
                                                     bool stash, float* pk)
    {
        const int RR = R > 0 ? R : Rrt;
        const int64_t e = base + o;
        float s = ld1(a.W[0] + e);
#pragma unroll
        for (int r = 1; r < RR; ++r) s = s + ld1(a.W[r] + e);
        const float u = ld1(a.Ur + e);
        const float wb = s * a.inv_R;
        const float v = wb + u;
        const float d = wb - v;
        const float dual_kept = u + d;
        st1(a.Z + e, kept ? v : (stash ? dual_kept : 0.f));
        st1(a.U + e, kept ? dual_kept : v);
        if (pk) pk[o] = v;
        if (a.Wbar) st1(a.Wbar + e, wb);
        return v;
    }
    // PARK forms (layers under both constraints): the candidate for the norms, the mean parked in Z, U untouched;
    // the outputs are written once both selections are known, from the parked mean and U
    static __device__ __forceinline__ double park_two(const ProjectArgs& a, int Rrt, int64_t e0, int64_t e1, double acc)
    {
        const int RR = R > 0 ? R : Rrt;
        v4f s0 = ld4(a.W[0] + e0), s1 = ld4(a.W[0] + e1);
#pragma unroll
        for (int r = 1; r < RR; ++r) {
            const v4f w0 = ld4(a.W[r] + e0), w1 = ld4(a.W[r] + e1);
            s0 = s0 + w0;
            s1 = s1 + w1;
        }
        const v4f u0 = ld4(a.Ur + e0), u1 = ld4(a.Ur + e1);
        const v4f wb0 = s0 * a.inv_R, wb1 = s1 * a.inv_R;
        st4(a.Z + e0, wb0);
        st4(a.Z + e1, wb1);
        acc = sq4(acc, wb0 + u0);
        return sq4(acc, wb1 + u1);
    }
    static __device__ __forceinline__ v4f park_one(const ProjectArgs& a, int Rrt, int64_t e)
    {
        const int RR = R > 0 ? R : Rrt;
        v4f s = ld4(a.W[0] + e);
#pragma unroll
        for (int r = 1; r < RR; ++r) s = s + ld4(a.W[r] + e);
        const v4f wb = s * a.inv_R;
        st4(a.Z + e, wb);
        return wb + ld4(a.Ur + e);
    }
    static __device__ __forceinline__ float park_scalar(const ProjectArgs& a, int Rrt, int64_t e)
    {
        const int RR = R > 0 ? R : Rrt;
        float s = ld1(a.W[0] + e);
#pragma unroll
        for (int r = 1; r < RR; ++r) s = s + ld1(a.W[r] + e);
        const float wb = s * a.inv_R;
        st1(a.Z + e, wb);
        return wb + ld1(a.Ur + e);
    }
    // the candidate alone; with park_mean the mean is parked in Z (CHANNEL layers: their outputs are written once
    // the mask is known, from the parked mean and U, so that the replicas are read once)
    static __device__ __forceinline__ v4f value4(const ProjectArgs& a, int Rrt, int64_t e)
    {
        const int RR = R > 0 ? R : Rrt;
        v4f s = ld4(a.W[0] + e);
#pragma unroll
        for (int r = 1; r < RR; ++r) s = s + ld4(a.W[r] + e);
        const v4f wb = s * a.inv_R;
        if (a.park_mean) st4(a.Z + e, wb);
        return wb + ld4(a.Ur + e);
    }
    static __device__ __forceinline__ float value1(const ProjectArgs& a, int Rrt, int64_t e)
    {
        const int RR = R > 0 ? R : Rrt;
        float s = ld1(a.W[0] + e);
#pragma unroll
        for (int r = 1; r < RR; ++r) s = s + ld1(a.W[r] + e);
        const float wb = s * a.inv_R;
        if (a.park_mean) st1(a.Z + e, wb);
        return wb + ld1(a.Ur + e);
    }
    static __device__ __forceinline__ float scalar(const ProjectArgs& a, int Rrt, int64_t e)
    {
        const int RR = R > 0 ? R : Rrt;
        float s = ld1(a.W[0] + e);
#pragma unroll
        for (int r = 1; r < RR; ++r) s = s + ld1(a.W[r] + e);
        const float u = ld1(a.Ur + e);
        const float wb = s * a.inv_R;
        const float v = wb + u;
        const float d = wb - v;
        st1(a.Z + e, v);
        st1(a.U + e, u + d);
        if (a.Wbar) st1(a.Wbar + e, wb);
        return v;
    }
};

// Sum of squares of the part of one row that lane j of `step` lanes owns (chunks j, j+step, ...),
// accumulated in increasing chunk order.
template <int R, bool PARK>
__device__ __forceinline__ double pass1_row(const ProjectArgs& a, int Rrt, int64_t base, int row_len, bool vec,
                                            int j, int step)
{
    double acc = 0.0;
    if (vec) {
        const int nchunk = row_len >> 2;
        int c = j;
        for (; c + step < nchunk; c += 2 * step) {
            const int64_t e0 = base + ((int64_t)c << 2), e1 = base + ((int64_t)(c + step) << 2);
            acc = PARK ? Cand<R>::park_two(a, Rrt, e0, e1, acc) : Cand<R>::two(a, Rrt, e0, e1, acc);
        }
        if (c < nchunk) {
            const int64_t e = base + ((int64_t)c << 2);
            acc = sq4(acc, PARK ? Cand<R>::park_one(a, Rrt, e) : Cand<R>::one(a, Rrt, e));
        }
    } else {
        for (int c = j; c < row_len; c += step) {
            const float v = PARK ? Cand<R>::park_scalar(a, Rrt, base + c) : Cand<R>::scalar(a, Rrt, base + c);
            acc = fma((double)v, (double)v, acc);
        }
    }
    return acc;
}

// FILTER / NONE: a group is a row.  Short rows: `lpr` <= 64 lanes share a row and a wave covers
// 64/lpr adjacent rows.  Long rows: the whole workgroup shares a row.  Per-lane sums are combined
// by a butterfly inside the wave and (long rows) in wave order through LDS, so the order of
// additions depends only on (row_len, lpr), never on where the row sits: equal groups get equal keys.
// PARK (layers under both constraints): the norms of the rows only; the mean goes to Z, U stays.
template <int R, bool PARK>
__device__ __forceinline__ void project_rows(const WorkItem& it, const ProjectArgs& a, int Rrt)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = it.row_len;
    const bool vec = item_vec(it);
    if (it.lpr <= kWave) {
        const int lpr = it.lpr;
        const int rpw = kWave / lpr;
        const int sub = lane / lpr;
        const int j = lane - sub * lpr;
        for (int rb = wave * rpw; rb < it.nr; rb += kWaves * rpw) {
            const int rr = rb + sub;
            const bool active = rr < it.nr;
            double acc = 0.0;
            if (active) acc = pass1_row<R, PARK>(a, Rrt, it.base + (int64_t)rr * row_len, row_len, vec, j, lpr);
            acc = wave_xor_sum(acc, lpr);
            if (active && j == 0) a.key[it.g0 + rr] = acc;
        }
    } else {
        __shared__ double wsum[kWaves];
        for (int rr = 0; rr < it.nr; ++rr) {
            double acc = pass1_row<R, PARK>(a, Rrt, it.base + (int64_t)rr * row_len, row_len, vec, threadIdx.x, kBlock);
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

// CHANNEL: a group is a block of khw adjacent columns of the [c_out][row_len] view.  A tile is
// (row block, column strip); each lane owns 4 (or 1) adjacent columns of the strip and walks down
// the rows of its wave, accumulating per-column sums in registers.  The four waves' sums are added
// in wave order through LDS and stored as this row block's partial column sums; the layer's selection later
// adds row blocks and the khw columns of a channel in a fixed order.
// No output is written speculatively: a pruned channel is a set of 4-byte (khw = 1) or 4*khw-byte runs
// scattered over every row, so repairing speculative outputs would rewrite most 128-bit quads of the
// layer.  Once the mask is known one streaming pass (channel_final) forms V = Wbar + U again, bit for bit, and
// writes the final Z and U: from the mean Wbar parked in Z here when there are 3 or more replicas (R + 6 arenas
// moved in all instead of 2R + 4), else from the replicas.
template <int R>
__device__ __forceinline__ void project_tile(const WorkItem& it, const ProjectArgs& a, int Rrt)
{
    __shared__ double part[kWaves][kWave * 4];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = it.row_len;
    const bool vec = item_vec(it);
    const int vw = vec ? 4 : 1;
    const int col = it.col0 + lane * vw;
    const bool in = col < row_len;
    double acc0 = 0.0, acc1 = 0.0, acc2 = 0.0, acc3 = 0.0;
    if (in) {
        int rr = wave;
        // Two of the wave's rows at a time (all their loads before the first store), summed in ascending order.  Not
        // with one replica or a replica count known only at run time: the registers this takes would lower the
        // occupancy of the kernel's other branches there.
        if constexpr (R >= 2) {
            if (vec) {
                auto finish4 = [&](int64_t e, const v4f& s, const v4f& u) {
                    const v4f wb = s * a.inv_R;
                    if (a.park_mean) st4(a.Z + e, wb);
                    const v4f v = wb + u;
                    acc0 = fma((double)v.x, (double)v.x, acc0);
                    acc1 = fma((double)v.y, (double)v.y, acc1);
                    acc2 = fma((double)v.z, (double)v.z, acc2);
                    acc3 = fma((double)v.w, (double)v.w, acc3);
                };
                for (; rr + kWaves < it.nr; rr += 2 * kWaves) {
                    const int64_t e0 = it.base + (int64_t)rr * row_len + col, e1 = e0 + (int64_t)kWaves * row_len;
                    v4f s0 = ld4(a.W[0] + e0), s1 = ld4(a.W[0] + e1);
#pragma unroll
                    for (int r = 1; r < R; ++r) {
                        const v4f w0 = ld4(a.W[r] + e0), w1 = ld4(a.W[r] + e1);
                        s0 = s0 + w0;
                        s1 = s1 + w1;
                    }
                    const v4f u0 = ld4(a.Ur + e0), u1 = ld4(a.Ur + e1);
                    finish4(e0, s0, u0);
                    finish4(e1, s1, u1);
                }
            }
        }
        for (; rr < it.nr; rr += kWaves) {
            const int64_t e = it.base + (int64_t)rr * row_len + col;
            if (vec) {
                const v4f v = Cand<R>::value4(a, Rrt, e);
                acc0 = fma((double)v.x, (double)v.x, acc0);
                acc1 = fma((double)v.y, (double)v.y, acc1);
                acc2 = fma((double)v.z, (double)v.z, acc2);
                acc3 = fma((double)v.w, (double)v.w, acc3);
            } else {
                const float v = Cand<R>::value1(a, Rrt, e);
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
        double* out = a.colpart + it.aux + col;
        for (int i = 0; i < vw; ++i) {
            double s = part[0][lane * 4 + i];
            for (int w = 1; w < kWaves; ++w) s += part[w][lane * 4 + i];
            out[i] = s;
        }
    }
}

template <int R>
__global__ __launch_bounds__(kBlock) void project_pass1(const WorkItem* __restrict__ items, ProjectArgs a, int Rrt)
{
    const WorkItem it = items[blockIdx.x];
    const int mode = item_mode(it);
    if (mode == HSADMM_MODE_CHANNEL) project_tile<R>(it, a, Rrt);
    else if (mode == HSADMM_MODE_BOTH) project_rows<R, true>(it, a, Rrt);       // the filter norms come first
    else project_rows<R, false>(it, a, Rrt);
}

// ------------------------------------------------------------------ project, pass 1 under a predicted selection

// The sparsity pattern stops changing after a few outer iterations (Section 4.5), so the selection of the previous
// iteration predicts this one's.  A selection record holds, for every group, its rank among the kept groups of its
// layer (what the compaction calls its position), or -1 if it was pruned.
struct HintArgs {
    const int32_t* sel_prev;   // groups_total: the previous selection's record
    float* packed;             // packed buffer of this call's compaction, or null (no compaction)
    int stash;                 // the dual is updated in place: rows predicted pruned keep the kept-form dual in Z
    int32_t* work;             // the work list the selection fills for the repair pass (pass 1 clears its counter)
    const DevLayer* layers;    // the plan's layer table
};

// pass1_row with the outputs of a row written in the form its prediction makes final (see Cand::put_h); the sum of
// squares is taken in the same order as there, so the keys carry the same bits.
template <int R>
__device__ __forceinline__ double pass1_row_hinted(const ProjectArgs& a, int Rrt, int64_t base, int row_len, bool vec,
                                                   int j, int step, bool kept, bool stash, float* pk)
{
    double acc = 0.0;
    if (vec) {
        const int nchunk = row_len >> 2;
        int c = j;
        for (; c + step < nchunk; c += 2 * step)
            acc = Cand<R>::two_h(a, Rrt, base, c << 2, (c + step) << 2, kept, stash, pk, acc);
        if (c < nchunk) acc = sq4(acc, Cand<R>::one_h(a, Rrt, base, c << 2, kept, stash, pk));
    } else {
        for (int c = j; c < row_len; c += step) {
            const float v = Cand<R>::scalar_h(a, Rrt, base, c, kept, stash, pk);
            acc = fma((double)v, (double)v, acc);
        }
    }
    return acc;
}

// project_rows for FILTER / NONE row items under a predicted selection.  A row predicted kept is written as pass 1
// always writes it and, with a compaction to follow, also at its predicted rank in the packed buffer; a row
// predicted pruned is written in its pruned form (see Cand::put_h).  The rows of an unconstrained layer are always
// kept, at their own index.  A rank outside [0, k) cannot have come from a selection of this plan: such a row is
// treated as kept and left for the repair pass to pack.
template <int R>
__device__ __forceinline__ void project_rows_hinted(const WorkItem& it, const ProjectArgs& a, int Rrt,
                                                    const HintArgs& h)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = it.row_len;
    const bool vec = item_vec(it);
    const bool unconstrained = item_mode(it) == HSADMM_MODE_NONE;
    const bool stash = h.stash != 0;
    float* const pk_layer = h.packed ? h.packed + it.packed_off : nullptr;
    auto prediction = [&](int rr, bool& kept, float*& pk) {
        const int hp = unconstrained ? it.row0 + rr : h.sel_prev[it.g0 + rr];
        kept = hp >= 0;
        pk = (pk_layer && kept && hp < it.k) ? pk_layer + (int64_t)hp * row_len : nullptr;
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
                float* pk;
                prediction(rr, kept, pk);
                acc = pass1_row_hinted<R>(a, Rrt, it.base + (int64_t)rr * row_len, row_len, vec, j, lpr, kept, stash, pk);
            }
            acc = wave_xor_sum(acc, lpr);
            if (active && j == 0) a.key[it.g0 + rr] = acc;
        }
    } else {
        __shared__ double wsum[kWaves];
        for (int rr = 0; rr < it.nr; ++rr) {
            bool kept;
            float* pk;
            prediction(rr, kept, pk);
            double acc = pass1_row_hinted<R>(a, Rrt, it.base + (int64_t)rr * row_len, row_len, vec, threadIdx.x, kBlock,
                                             kept, stash, pk);
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

// project_tile under a predicted selection, for a dual written out of place: besides the column sums, the tile's
// elements are written in the final form the prediction gives them -- Z <- V in the columns of channels predicted
// kept, +0 in the others, the updated dual U + (Wbar - Z), and, with a compaction, the kept columns at their
// predicted place in the packed row.  If the selection then keeps exactly the predicted channels the layer is
// done; otherwise the repair pass forms the layer again from the replicas and the old dual, which is still there.
// A lane's four columns keep their flags and packed columns for the whole tile.
// WEIGHTED: the candidate is z~ = fl(fl(a t) + fl(b (Zg - Vd))), t = Wbar + U (Eq. (9)); the column sums are those of
// z~ and what is packed is c = z + Vd (Section 4.4.1).
template <int R, bool WEIGHTED = false>
__device__ __forceinline__ void project_tile_hinted(const WorkItem& it, const ProjectArgs& a, int Rrt, const HintArgs& h)
{
    __shared__ double part[kWaves][kWave * 4];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = it.row_len;
    const bool vec = item_vec(it);
    const int vw = vec ? 4 : 1;
    const int col = it.col0 + lane * vw;
    const bool in = col < row_len;
    const int khw = it.khw;
    const int packed_row_len = it.k * khw;
    double acc0 = 0.0, acc1 = 0.0, acc2 = 0.0, acc3 = 0.0;
    if (in) {
        bool kept[4] = {false, false, false, false};
        int pc[4] = {-1, -1, -1, -1};            // packed column, -1: not packed here
        const DivKhw div(khw);
        const int32_t* hp_l = h.sel_prev + it.g0;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            if (i < vw) {
                const int ch = div(col + i);
                const int hp = hp_l[ch];
                kept[i] = hp >= 0;
                if (h.packed && hp >= 0 && hp < it.k) pc[i] = hp * khw + (col + i - ch * khw);
            }
        }
        float* const pk_layer = h.packed ? h.packed + it.packed_off : nullptr;
        const int RR = R > 0 ? R : Rrt;
        const float al = WEIGHTED ? a.coef[2 * it.layer] : 1.f, bl = WEIGHTED ? a.coef[2 * it.layer + 1] : 0.f;
        // the outputs of one row's quad and its share of the column sums
        auto finish4 = [&](int rr, int64_t e, const v4f& s, const v4f& u) {
            float* drow = pk_layer ? pk_layer + (int64_t)(it.row0 + rr) * packed_row_len : nullptr;
            const v4f wb = s * a.inv_R;
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
            z.x = kept[0] ? v.x : 0.f; z.y = kept[1] ? v.y : 0.f; z.z = kept[2] ? v.z : 0.f; z.w = kept[3] ? v.w : 0.f;
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
            acc0 = fma((double)v.x, (double)v.x, acc0);
            acc1 = fma((double)v.y, (double)v.y, acc1);
            acc2 = fma((double)v.z, (double)v.z, acc2);
            acc3 = fma((double)v.w, (double)v.w, acc3);
        };
        if (vec) {
            int rr = wave;
            // two of the wave's rows at a time (all their loads before the first store), in ascending order
            for (; rr + kWaves < it.nr; rr += 2 * kWaves) {
                const int64_t e0 = it.base + (int64_t)rr * row_len + col, e1 = e0 + (int64_t)kWaves * row_len;
                v4f s0 = ld4(a.W[0] + e0), s1 = ld4(a.W[0] + e1);
#pragma unroll
                for (int r = 1; r < RR; ++r) {
                    const v4f w0 = ld4(a.W[r] + e0), w1 = ld4(a.W[r] + e1);
                    s0 = s0 + w0;
                    s1 = s1 + w1;
                }
                const v4f u0 = ld4(a.Ur + e0), u1 = ld4(a.Ur + e1);
                finish4(rr, e0, s0, u0);
                finish4(rr + kWaves, e1, s1, u1);
            }
            if (rr < it.nr) {
                const int64_t e = it.base + (int64_t)rr * row_len + col;
                v4f s = ld4(a.W[0] + e);
#pragma unroll
                for (int r = 1; r < RR; ++r) s = s + ld4(a.W[r] + e);
                const v4f u = ld4(a.Ur + e);
                finish4(rr, e, s, u);
            }
        } else {
            for (int rr = wave; rr < it.nr; rr += kWaves) {
                const int64_t e = it.base + (int64_t)rr * row_len + col;
                float* drow = pk_layer ? pk_layer + (int64_t)(it.row0 + rr) * packed_row_len : nullptr;
                float s = ld1(a.W[0] + e);
#pragma unroll
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
                const float z = kept[0] ? v : 0.f;
                st1(a.Z + e, z);
                st1(a.U + e, u + (wb - z));
                if (a.Wbar) st1(a.Wbar + e, wb);
                if (drow && pc[0] >= 0) drow[pc[0]] = WEIGHTED ? z + vd : z;
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
        double* out = a.colpart + it.aux + col;
        for (int i = 0; i < vw; ++i) {
            double s = part[0][lane * 4 + i];
            for (int w = 1; w < kWaves; ++w) s += part[w][lane * 4 + i];
            out[i] = s;
        }
    }
}

// ------------------------------------------------------------------ BOTH: channel norms after the filter projection

// Second projection of a layer under both constraints (Section 3, paragraph after Eq. (10)): the
// channel norms of the tensor whose pruned filters are already zero, i.e. column sums of V^2 over
// the kept rows only.  After pass 1 Z holds the mean and the candidate is formed again, bit for bit: V = Z + U, or,
// for the weighted projection (coef given), z~ = fl(fl(a (Z + U)) + fl(b (Zg - Vd))).  Tiles and the order of
// additions are those of project_tile (rows of a pruned filter add nothing and are not read).
__global__ __launch_bounds__(kBlock) void composite_colsums(const WorkItem* __restrict__ items,
                                                            const float* __restrict__ Z,
                                                            const float* __restrict__ U,
                                                            const float* __restrict__ Zg,
                                                            const float* __restrict__ Vd,
                                                            const float* __restrict__ coef,
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
    const uint8_t* mf = mask + it.g0 + it.row0;      // filter bytes of the tile's rows
    const float al = coef ? coef[2 * it.layer] : 1.f, bl = coef ? coef[2 * it.layer + 1] : 0.f;
    double acc0 = 0.0, acc1 = 0.0, acc2 = 0.0, acc3 = 0.0;
    if (in) {
        for (int rr = wave; rr < it.nr; rr += kWaves) {
            if (mf[rr] == 0) continue;
            const int64_t e = it.base + (int64_t)rr * row_len + col;
            if (vec) {
                v4f v = ld4(Z + e) + ld4(U + e);
                if (coef) {
                    const v4f q = ld4(Zg + e) - ld4(Vd + e);
                    const v4f at = v * al;
                    const v4f bq = q * bl;
                    v = at + bq;
                }
                acc0 = fma((double)v.x, (double)v.x, acc0);
                acc1 = fma((double)v.y, (double)v.y, acc1);
                acc2 = fma((double)v.z, (double)v.z, acc2);
                acc3 = fma((double)v.w, (double)v.w, acc3);
            } else {
                float v = ld1(Z + e) + ld1(U + e);
                if (coef) {
                    const float q = ld1(Zg + e) - ld1(Vd + e);
                    const float at = v * al;
                    const float bq = q * bl;
                    v = at + bq;
                }
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


// ------------------------------------------------------------------ project, fix-up of pruned groups

// pr[i] = the channel of column col + i is pruned (mc: the layer's channel bytes), for 4 adjacent columns.
__device__ __forceinline__ void quad_pruned(const uint8_t* __restrict__ mc, const DivKhw& div, int col, bool pr[4])
{
    if (div.khw == 1) {
        unsigned int m4;
        __builtin_memcpy(&m4, mc + col, 4);
#pragma unroll
        for (int i = 0; i < 4; ++i) pr[i] = ((m4 >> (8 * i)) & 0xffu) == 0u;
    } else if (div.khw >= 4) {
        // at most two channels meet in a quad
        const int ch = div(col);
        const int left = (ch + 1) * div.khw - col;          // columns of the quad that belong to ch
        const bool p0 = mc[ch] == 0;
        const bool p1 = left < 4 ? mc[ch + 1] == 0 : p0;
#pragma unroll
        for (int i = 0; i < 4; ++i) pr[i] = i < left ? p0 : p1;
    } else {
#pragma unroll
        for (int i = 0; i < 4; ++i) pr[i] = mc[div(col + i)] == 0;
    }
}

// Row items of the FILTER layers.  A pruned filter's row moves whole: U <- V (held in Z), Z <- +0; kept rows are
// final already.
__device__ __forceinline__ void fixup_rows(const WorkItem& it, const uint8_t* mask, float* U, float* Z)
{
    const int row_len = it.row_len;
    const bool vec = item_vec(it);
    const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
    // lanes-per-row mapping as in pass 1 (the mapping carries no arithmetic here)
    const int lpr = it.lpr <= kWave ? it.lpr : kBlock;
    const int rows_at_once = kBlock / lpr;
    const int sub = threadIdx.x / lpr;
    const int j = threadIdx.x - sub * lpr;
    for (int rr = sub; rr < it.nr; rr += rows_at_once) {
        if (mask[it.g0 + rr] != 0) continue;
        const int64_t base = it.base + (int64_t)rr * row_len;
        if (vec) {
            const int nchunk = row_len >> 2;
            for (int c = j; c < nchunk; c += lpr) {
                const int64_t e = base + ((int64_t)c << 2);
                st4(U + e, ld4(Z + e));
                st4(Z + e, zero4);
            }
        } else {
            for (int c = j; c < row_len; c += lpr) {
                st1(U + base + c, ld1(Z + base + c));
                st1(Z + base + c, 0.f);
            }
        }
    }
}

__global__ __launch_bounds__(kBlock) void project_fixup(const WorkItem* __restrict__ items,
                                                        const uint8_t* __restrict__ mask,
                                                        float* __restrict__ U, float* __restrict__ Z)
{
    fixup_rows(items[blockIdx.x], mask, U, Z);
}


}  // namespace
#endif
