// hsadmm_residuals: layer-wise squared residual norms in fp64.
// Part of the single translation unit built from hsadmm.hip (included there, in order).
#ifndef KERNELS_RESIDUALS_HPP
#define KERNELS_RESIDUALS_HPP
#include "hsadmm_device.hpp"

namespace {

// ------------------------------------------------------------------ residual norms (Algorithm 1 Phase 5)

struct ResidualArgs {
    const float* W[HSADMM_MAX_REPLICAS];
    const float* Zi;
    const float* Zi_prev;   // may be null
    const float* Zg;        // may be null
    const float* Zg_prev;   // may be null
    double* part;           // per row item: 4 partial sums
};

// One workgroup per row item (a contiguous span of one layer): per-thread fp64 sums of the four
// squared differences, combined by a butterfly per wave and in wave order through LDS.
// modes: bit m set = the items of layers of mode m are processed (the others return at once and leave their
// partial sums alone).
template <int R>
__global__ __launch_bounds__(kBlock) void residual_partials(const WorkItem* __restrict__ items, ResidualArgs a, int Rrt,
                                                            int modes)
{
    __shared__ double red[kWaves][4];
    const int RR = R > 0 ? R : Rrt;
    const WorkItem it = items[blockIdx.x];
    if (((modes >> item_mode(it)) & 1) == 0) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int64_t len = (int64_t)it.nr * it.row_len;
    double s0 = 0.0, s1 = 0.0, s2 = 0.0, s3 = 0.0;
    if (item_vec(it)) {
        for (int64_t c = threadIdx.x; c < (len >> 2); c += kBlock) {
            const int64_t e = it.base + (c << 2);
            const v4f zi = ld4(a.Zi + e);
#pragma unroll
            for (int r = 0; r < RR; ++r) {
                const v4f w = ld4(a.W[r] + e);
                s0 = sqd(s0, w.x, zi.x); s0 = sqd(s0, w.y, zi.y); s0 = sqd(s0, w.z, zi.z); s0 = sqd(s0, w.w, zi.w);
            }
            if (a.Zi_prev) {
                const v4f p = ld4(a.Zi_prev + e);
                s1 = sqd(s1, zi.x, p.x); s1 = sqd(s1, zi.y, p.y); s1 = sqd(s1, zi.z, p.z); s1 = sqd(s1, zi.w, p.w);
            }
            if (a.Zg) {
                const v4f g = ld4(a.Zg + e);
                s2 = sqd(s2, zi.x, g.x); s2 = sqd(s2, zi.y, g.y); s2 = sqd(s2, zi.z, g.z); s2 = sqd(s2, zi.w, g.w);
                if (a.Zg_prev) {
                    const v4f q = ld4(a.Zg_prev + e);
                    s3 = sqd(s3, g.x, q.x); s3 = sqd(s3, g.y, q.y); s3 = sqd(s3, g.z, q.z); s3 = sqd(s3, g.w, q.w);
                }
            }
        }
    } else {
        for (int64_t c = threadIdx.x; c < len; c += kBlock) {
            const int64_t e = it.base + c;
            const float zi = a.Zi[e];
            for (int r = 0; r < RR; ++r) s0 = sqd(s0, a.W[r][e], zi);
            if (a.Zi_prev) s1 = sqd(s1, zi, a.Zi_prev[e]);
            if (a.Zg) {
                s2 = sqd(s2, zi, a.Zg[e]);
                if (a.Zg_prev) s3 = sqd(s3, a.Zg[e], a.Zg_prev[e]);
            }
        }
    }
    s0 = wave_xor_sum(s0, kWave); s1 = wave_xor_sum(s1, kWave);
    s2 = wave_xor_sum(s2, kWave); s3 = wave_xor_sum(s3, kWave);
    if (lane == 0) { red[wave][0] = s0; red[wave][1] = s1; red[wave][2] = s2; red[wave][3] = s3; }
    __syncthreads();
    if (threadIdx.x < 4) {
        double t = red[0][threadIdx.x];
        for (int w = 1; w < kWaves; ++w) t += red[w][threadIdx.x];
        a.part[(int64_t)blockIdx.x * 4 + threadIdx.x] = t;
    }
}

// Squared norm of one arena per row item, in fp64: part[4 * item] (the other three slots of the item are left alone).
// Same per-thread strides and the same order of combination as residual_partials.
__global__ __launch_bounds__(kBlock) void sqnorm_partials(const WorkItem* __restrict__ items, const float* __restrict__ X,
                                                          double* __restrict__ part)
{
    __shared__ double red[kWaves];
    const WorkItem it = items[blockIdx.x];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int64_t len = (int64_t)it.nr * it.row_len;
    double s = 0.0;
    if (item_vec(it)) {
        for (int64_t c = threadIdx.x; c < (len >> 2); c += kBlock) {
            const v4f x = ld4(X + it.base + (c << 2));
            s = fma((double)x.x, (double)x.x, s);
            s = fma((double)x.y, (double)x.y, s);
            s = fma((double)x.z, (double)x.z, s);
            s = fma((double)x.w, (double)x.w, s);
        }
    } else {
        for (int64_t c = threadIdx.x; c < len; c += kBlock) {
            const double x = (double)X[it.base + c];
            s = fma(x, x, s);
        }
    }
    s = wave_xor_sum(s, kWave);
    if (lane == 0) red[wave] = s;
    __syncthreads();
    if (threadIdx.x == 0) {
        double t = red[0];
        for (int w = 1; w < kWaves; ++w) t += red[w];
        part[(int64_t)blockIdx.x * 4] = t;
    }
}

// One workgroup per layer: adds the layer's item partials (thread t takes items t, t+256, ... in
// order; threads are combined by a butterfly per wave and in wave order), writes out[k*L + l] for the
// norms k0 <= k < k1 (the others are neither read nor written).
__global__ __launch_bounds__(kBlock) void residual_finish(const DevLayer* __restrict__ layers, int nL,
                                                          const double* __restrict__ part, double* __restrict__ out,
                                                          int k0, int k1)
{
    __shared__ double red[kWaves][4];
    const int l = blockIdx.x;
    const int first = layers[l].rows_item0, count = layers[l].rows_items;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    double s[4] = {0.0, 0.0, 0.0, 0.0};
    for (int i = threadIdx.x; i < count; i += kBlock)
#pragma unroll
        for (int k = 0; k < 4; ++k)
            if (k >= k0 && k < k1) s[k] += part[(int64_t)(first + i) * 4 + k];
    for (int k = 0; k < 4; ++k) s[k] = wave_xor_sum(s[k], kWave);
    if (lane == 0) for (int k = 0; k < 4; ++k) red[wave][k] = s[k];
    __syncthreads();
    if ((int)threadIdx.x >= k0 && (int)threadIdx.x < k1) {
        double t = red[0][threadIdx.x];
        for (int w = 1; w < kWaves; ++w) t += red[w][threadIdx.x];
        out[(int64_t)threadIdx.x * nL + l] = t;
    }
}

// Rows 0 and 1 of the residual norms of the CHANNEL and BOTH layers after a dynamic projection that took the norms
// on the way (the selection itself finishes the FILTER and unconstrained layers): one workgroup per layer adds the
// partial sums of the layer's row items, as residual_finish does; workgroups of other layers return at once.
__global__ __launch_bounds__(kBlock) void residual_pick(const DevLayer* __restrict__ layers, int nL,
                                                        const double* __restrict__ part, double* __restrict__ out)
{
    __shared__ double red[kWaves][2];
    const int l = blockIdx.x;
    const DevLayer L = layers[l];
    if (L.mode == HSADMM_MODE_FILTER || L.mode == HSADMM_MODE_NONE) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    double s0 = 0.0, s1 = 0.0;
    for (int i = threadIdx.x; i < L.rows_items; i += kBlock) {
        s0 += part[(int64_t)(L.rows_item0 + i) * 4 + 0];
        s1 += part[(int64_t)(L.rows_item0 + i) * 4 + 1];
    }
    s0 = wave_xor_sum(s0, kWave);
    s1 = wave_xor_sum(s1, kWave);
    if (lane == 0) { red[wave][0] = s0; red[wave][1] = s1; }
    __syncthreads();
    if (threadIdx.x < 2) {
        double t = red[0][threadIdx.x];
        for (int w = 1; w < kWaves; ++w) t += red[w][threadIdx.x];
        out[(int64_t)threadIdx.x * nL + l] = t;
    }
}

}  // namespace
#endif
