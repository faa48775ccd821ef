// The un-predicted projection with a prediction formed inside the call (FILTER and unconstrained layers, dual in
// place): pass 1 holds a row item's outputs back in LDS until the item's keys are complete and then writes every row
// in the form its key suggests, given an estimate of the layer's selection threshold from the keys of the layer's
// first rows, which are processed ahead of the rest.  A prediction only chooses the form a row is written in; the
// selection and the repair pass after it give every output its exact value whatever was predicted (Eq. (10), Eq. (12)).
// Part of the single translation unit built from hsadmm.hip (included there, in order).
#ifndef KERNELS_ESTIMATE_HPP
#define KERNELS_ESTIMATE_HPP
#include "hsadmm_device.hpp"
#include "kernels_project.hpp"

namespace {

constexpr int kStageElems = 4608;       // elements of a row item that can be held back (two floats each: 36 KB of LDS)
constexpr int kStageRows = 64;          // ... and its rows
constexpr int kSampleKeys = 128;        // keys of a layer's first rows that the estimate is made of, at most
constexpr long long kEstimateMinElems = 20ll << 20;   // plans smaller than this keep the plain pass 1
constexpr int kKeptNoRank = 0x7fffffff; // a prediction record's entry for "kept, at a rank not known yet"
// WorkItem.col0 of a row item in the estimate's item order
constexpr int kEstPlain = 0;            // written as ever (unconstrained layers; items that cannot be held back)
constexpr int kEstSample = 1;           // one of a FILTER layer's first items: default form, its keys are published
constexpr int kEstUse = 2;              // a later item of a FILTER layer: form by the estimate

// Rows at the head of a layer of G groups whose keys make the estimate: a sixteenth, 16 at least, kSampleKeys at most
// (whole work items: a few more where the last of them reaches further).
__host__ __device__ __forceinline__ int sample_rows_of(int G)
{
    const int s = (G + 15) / 16;
    return s < 16 ? 16 : (s > kSampleKeys ? kSampleKeys : s);
}

struct EstArgs {
    int32_t* pred;          // groups_total: the form every FILTER row was written in (kKeptNoRank or -1), read by the repair
    unsigned int* tag;      // per layer, per sample row: the number of the call that published the row's key
    double* keys;           // per layer: the keys of its first kSampleKeys rows, as far as published
    double* thr;            // per layer: the threshold estimated from them ...
    unsigned int* thr_tag;  // ... and the number of the call that estimated it
    const DevLayer* layers;
    unsigned int gen;       // this call's number: keys tagged by another call are not this call's
};

__device__ __forceinline__ void lds_st4(float* p, const v4f& v) { *reinterpret_cast<v4f*>(p) = v; }
__device__ __forceinline__ v4f lds_ld4(const float* p) { return *reinterpret_cast<const v4f*>(p); }

// pass1_row with the candidate and the kept-form dual of every chunk going to LDS (sv, sd: the row's place there)
// instead of Z and U; the same loads, arithmetic and order of additions.
template <int R>
__device__ __forceinline__ double pass1_row_staged(const ProjectArgs& a, int Rrt, int64_t base, int row_len, int j,
                                                   int step, float* sv, float* sd)
{
    const int RR = R > 0 ? R : Rrt;
    double acc = 0.0;
    const int nchunk = row_len >> 2;
    int c = j;
    for (; c + step < nchunk; c += 2 * step) {
        const int o0 = c << 2, o1 = (c + step) << 2;
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
        lds_st4(sv + o0, v0);
        lds_st4(sv + o1, v1);
        lds_st4(sd + o0, u0 + d0);
        lds_st4(sd + o1, u1 + d1);
        if (a.Wbar) { st4(a.Wbar + e0, wb0); st4(a.Wbar + e1, wb1); }
        acc = sq4(acc, v0);
        acc = sq4(acc, v1);
    }
    if (c < nchunk) {
        const int o = c << 2;
        const int64_t e = base + o;
        v4f s = ld4(a.W[0] + e);
#pragma unroll
        for (int r = 1; r < RR; ++r) s = s + ld4(a.W[r] + e);
        const v4f u = ld4(a.Ur + e);
        const v4f wb = s * a.inv_R;
        const v4f v = wb + u;
        const v4f d = wb - v;
        lds_st4(sv + o, v);
        lds_st4(sd + o, u + d);
        if (a.Wbar) st4(a.Wbar + e, wb);
        acc = sq4(acc, v);
    }
    return acc;
}

// The key of row `row` (< kSampleKeys) of layer l for this call's estimate: a slot of its own, tagged with the call's
// number, so nothing is counted and nothing has to be cleared between calls.
__device__ __forceinline__ void publish_key(const EstArgs& x, int l, int row, double key)
{
    if (row >= kSampleKeys) return;
    // device-scope stores: the readers run on other compute units, behind other L2 caches
    __hip_atomic_store(&x.keys[(int64_t)l * kSampleKeys + row], key, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __hip_atomic_store(&x.tag[(int64_t)l * kSampleKeys + row], x.gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}

// Run by a workgroup that has just published keys of layer l: the estimate of the layer's threshold from all keys
// published so far in this call -- with m of them and the layer keeping k of G groups, the key that r = round(m k / G)
// of the m exceed, so that about k / G of the layer's keys lie above it -- published in turn (the workgroup that
// finishes last among those of the layer's first rows leaves the estimate made of all of them).  sk: kSampleKeys
// doubles of LDS.  A key that is being written while it is read here gives a worse estimate, never a wrong result.
__device__ __forceinline__ void publish_threshold(const EstArgs& x, int l, double* sk)
{
    const int t = threadIdx.x;
    bool valid = false;
    double mine = -1.0;                                          // (keys are sums of squares: an empty slot ranks last)
    if (t < kSampleKeys) {
        const unsigned int tag = __hip_atomic_load(&x.tag[(int64_t)l * kSampleKeys + t], __ATOMIC_RELAXED,
                                                   __HIP_MEMORY_SCOPE_AGENT);
        const double key = __hip_atomic_load(&x.keys[(int64_t)l * kSampleKeys + t], __ATOMIC_RELAXED,
                                             __HIP_MEMORY_SCOPE_AGENT);
        valid = tag == x.gen && key >= 0.0;
        if (valid) mine = key;
        sk[t] = mine;
    }
    const int m = __syncthreads_count(valid ? 1 : 0);            // (also: sk is complete)
    const DevLayer& L = x.layers[l];
    // only a workgroup that finds all of the layer's first rows published goes on: the last to arrive (it looks
    // after the barrier that follows its own stores; should two that finish together both miss each other's keys,
    // the layer gets no estimate in this call and its rows take the likelier form, as before any estimate exists)
    const int expected = min(sample_rows_of(L.G), L.G);
    if (m < 8 || m < expected) return;
    const int r = (int)(((long long)m * L.k + L.G / 2) / L.G);
    bool winner = false;
    double thr = -1.0;                                           // r >= m: every key lies above
    if (r >= m) {
        winner = t == 0;
    } else if (t < kSampleKeys) {
        int above = 0, equal_before = 0;
        for (int i0 = 0; i0 < kSampleKeys; i0 += 16) {
            double o[16];                                        // sixteen LDS reads in flight
#pragma unroll
            for (int i = 0; i < 16; ++i) o[i] = sk[i0 + i];
#pragma unroll
            for (int i = 0; i < 16; ++i) {
                above += o[i] > mine ? 1 : 0;
                equal_before += (o[i] == mine && i0 + i < t) ? 1 : 0;
            }
        }
        winner = above + equal_before == r;                      // ranks are a permutation: exactly one key has rank r
        thr = mine;
    }
    if (winner) {
        __hip_atomic_store(&x.thr[l], thr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        __hip_atomic_store(&x.thr_tag[l], x.gen, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
}

// project_rows for a FILTER row item of at most kStageElems elements and kStageRows rows, rows a multiple of 4 floats
// long: keys as there; the outputs wait in LDS and are written once every row of the item has its key, a row predicted
// kept as Z <- V, U <- the kept-form dual, a row predicted pruned with the two changed over (U <- V is final if it is
// pruned, Z keeps the kept-form dual for the repair pass, as under a caller's prediction with the dual in place).
template <int R>
__device__ __forceinline__ void project_rows_staged(const WorkItem& it, const ProjectArgs& a, int Rrt, const EstArgs& x,
                                                    float* stage, double* skey, unsigned char* sform, double* sk,
                                                    double* sthr)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = it.row_len;
    const int n_elems = it.nr * row_len;
    float* const sV = stage;
    float* const sD = stage + kStageElems;
    // the layer's estimate as it stands now (asked for ahead of the rows, so that it costs no wait of its own)
    unsigned int thr_tag = 0;
    double thr_val = 0.0;
    if (it.col0 == kEstUse && threadIdx.x == 0) {
        thr_tag = __hip_atomic_load(&x.thr_tag[it.layer], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
        thr_val = __hip_atomic_load(&x.thr[it.layer], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    if (it.lpr <= kWave) {
        const int lpr = it.lpr;
        const int rpw = kWave / lpr;
        const int sub = lane / lpr;
        const int j = lane - sub * lpr;
        for (int rb = wave * rpw; rb < it.nr; rb += kWaves * rpw) {
            const int rr = rb + sub;
            const bool active = rr < it.nr;
            double acc = 0.0;
            if (active)
                acc = pass1_row_staged<R>(a, Rrt, it.base + (int64_t)rr * row_len, row_len, j, lpr, sV + rr * row_len,
                                          sD + rr * row_len);
            acc = wave_xor_sum(acc, lpr);
            if (active && j == 0) { a.key[it.g0 + rr] = acc; skey[rr] = acc; }
        }
    } else {
        __shared__ double wsum[kWaves];
        for (int rr = 0; rr < it.nr; ++rr) {
            double acc = pass1_row_staged<R>(a, Rrt, it.base + (int64_t)rr * row_len, row_len, threadIdx.x, kBlock,
                                             sV + rr * row_len, sD + rr * row_len);
            acc = wave_xor_sum(acc, kWave);
            if (lane == 0) wsum[wave] = acc;
            __syncthreads();
            if (threadIdx.x == 0) {
                double s = wsum[0];
                for (int w = 1; w < kWaves; ++w) s += wsum[w];
                a.key[it.g0 + rr] = s;
                skey[rr] = s;
            }
            __syncthreads();
        }
    }
    __syncthreads();
    // the form of every row: by the layer's estimate where there is one already, else the likelier outcome
    const DevLayer& L = x.layers[it.layer];
    const bool kept_default = 2 * L.k >= L.G;
    if (it.col0 == kEstUse) {
        if (threadIdx.x == 0) {
            if (thr_tag != x.gen) {                              // not there when this item began: one more look
                thr_tag = __hip_atomic_load(&x.thr_tag[it.layer], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                thr_val = __hip_atomic_load(&x.thr[it.layer], __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            }
            sthr[0] = thr_val;
            sthr[1] = thr_tag == x.gen ? 1.0 : 0.0;
        }
        __syncthreads();
    } else {
        for (int rr = threadIdx.x; rr < it.nr; rr += kBlock) publish_key(x, it.layer, it.row0 + rr, skey[rr]);
        __syncthreads();
        publish_threshold(x, it.layer, sk);
    }
    const bool have = it.col0 == kEstUse && sthr[1] != 0.0;
    const double thr = have ? sthr[0] : 0.0;
    for (int rr = threadIdx.x; rr < it.nr; rr += kBlock) {
        const bool kept = have ? skey[rr] > thr : kept_default;
        sform[rr] = kept ? 1 : 0;
        x.pred[it.g0 + rr] = kept ? kKeptNoRank : -1;
    }
    __syncthreads();
    const DivKhw row_of(row_len >> 2);                           // (chunks per row)
    for (int q = threadIdx.x; q < (n_elems >> 2); q += kBlock) {
        const bool kept = sform[row_of(q)] != 0;
        const v4f v = lds_ld4(sV + 4 * q), d = lds_ld4(sD + 4 * q);
        const int64_t e = it.base + 4 * (int64_t)q;
        st4(a.Z + e, kept ? v : d);
        st4(a.U + e, kept ? d : v);
    }
}

// Pass 1 of a plan of FILTER and unconstrained layers with the prediction formed inside the call.  Items come in the
// estimate's order (every FILTER layer's first items ahead of all others).
template <int R>
__global__ __launch_bounds__(kBlock) void project_pass1_est(const WorkItem* __restrict__ items, ProjectArgs a, int Rrt,
                                                            EstArgs x)
{
    __shared__ __align__(16) float stage[2 * kStageElems];
    __shared__ double skey[kStageRows];
    __shared__ double sk[kSampleKeys];
    __shared__ double sthr[2];
    __shared__ unsigned char sform[kStageRows];
    const WorkItem it = items[blockIdx.x];
    if (it.col0 != kEstPlain) {
        project_rows_staged<R>(it, a, Rrt, x, stage, skey, sform, sk, sthr);
    } else {
        project_rows<R, false>(it, a, Rrt);                      // kept form, as ever
        if (item_mode(it) == HSADMM_MODE_FILTER)
            for (int rr = threadIdx.x; rr < it.nr; rr += kBlock) x.pred[it.g0 + rr] = kKeptNoRank;
    }
}

}  // namespace
#endif
