// HIP kernels (gfx950 / CDNA4) and C ABI of the H-SADMM structured-sparsity step.
// The interface, data layout and arithmetic contract are stated in include/hsadmm.h.
//
// Kernel overview (every launch covers all layers of the plan through a work-item table):
//
//   project_pass1   streams the R replicas and U once.  Computes Wbar, V = Wbar + U, the fp64
//                   partial sums of V^2, and writes the values that are final if the group is
//                   kept: Z <- V, U <- U + (Wbar - V).                       [Eq. (9), (12)]
//   select_topk     one workgroup per layer: byte-wise radix select of the k-th largest key on
//                   the uint64 view of the non-negative doubles (bytes all keys share are skipped,
//                   the search stops once one candidate is left), ties cut by an ordered scan so
//                   that lower indices win.                                  [Eq. (10)]
//   project_fixup   touches pruned groups only: U <- V (taken from Z), Z <- +0.  For a pruned
//                   group U + (Wbar - 0) equals V bit for bit, so no replica is read again.
//   scan_mask       per layer: kept count, exclusive positions, kept_idx, layer_off.
//   compact_gather  packed <- src[K_out, K_in, :]                             [Eq. (15)]
//   expand_scatter  dst <- zero fill + scatter of packed                      [Section 4.4.3]
//
// Nothing here is a dense contraction, so no MFMA is used; every kernel is bound by HBM traffic.
// Arena data is touched once per kernel, so it is moved with non-temporal 128-bit accesses.
// fp32 arithmetic is compiled without contraction (-ffp-contract=off); the fp64 accumulation
// uses fma(v, v, acc), which equals mul+add because the square of an fp32 value is exact in fp64.

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstdint>
#include <cstdlib>
#include <cstring>
#include <new>
#include <vector>

#include "hsadmm.h"

namespace {

constexpr int kWave = 64;
constexpr int kBlock = 256;                 // streaming kernels: 4 waves
constexpr int kWaves = kBlock / kWave;
constexpr int kScanBlock = 1024;            // select_topk and scan_mask
constexpr int kScanWaves = kScanBlock / kWave;
constexpr int kTileElems = 2048;                // target elements per work item
constexpr int kWideRow = 2048;                  // rows at least this long are shared by the whole workgroup
constexpr int kChanRows = 32;               // CHANNEL tiles: rows per row block
constexpr int kTopkRegs = 8;                // the selection keeps up to 8 keys per thread in registers
constexpr int kVersion = 130;

typedef float v4f __attribute__((ext_vector_type(4)));

struct DevLayer {
    int64_t elem_off;
    int64_t colpart_off;    // CHANNEL: first double of this layer's per-row-block column sums
    int64_t unit;           // packed elements one kept group contributes (NONE: the whole layer)
    int32_t c_out, c_in, khw, mode, k;
    int32_t G, group_base, row_len;
    int32_t n_rowblocks;    // CHANNEL: ceil(c_out / kChanRows)
    int32_t rows_item0;     // first of this layer's row items (compact / expand / residual kernels)
    int32_t rows_items;     // number of them
    int32_t pad_;
};

// One unit of work for a 256-thread workgroup; it carries everything the streaming kernels need,
// so a workgroup starts with a single 64-byte scalar load.
//   row item  (FILTER / NONE in project kernels, every mode in compact / expand): rows [r0, r0+nr)
//   tile item (CHANNEL in project kernels): rows [r0, r0+nr) x one column strip
struct WorkItem {
    int64_t base;       // arena element offset of the item's first row (column 0)
    int64_t aux;        // tile: offset (doubles) of this row block's column sums in the workspace
    int32_t g0;         // row item: index in mask/key/pos of the first row; tile: group_base
    int32_t nr;         // rows
    int32_t row_len;    // c_in * khw
    int32_t lpr;        // row item: lanes sharing a row, power of two <= 64, or 256 (whole workgroup)
    int32_t flags;      // bits 0-1: mode; bit 2: 128-bit path (row_len % 4 == 0)
    int32_t col0;       // tile: first column of the strip; CHANNEL row item: index of the first row
    int32_t khw;
    int32_t layer;
    int32_t pad_[4];
};
static_assert(sizeof(WorkItem) == 64, "WorkItem layout");

__device__ __forceinline__ int item_mode(const WorkItem& it) { return it.flags & 3; }
__device__ __forceinline__ bool item_vec(const WorkItem& it) { return (it.flags & 4) != 0; }

struct ProjectArgs {
    const float* W[HSADMM_MAX_REPLICAS];
    float* U;
    float* Z;
    float* Wbar;      // may be null
    double* key;      // groups_total
    double* colpart;  // CHANNEL partial column sums
    float inv_R;
};

// Streaming (touch-once) accesses.
__device__ __forceinline__ v4f ld4(const float* p) { return __builtin_nontemporal_load(reinterpret_cast<const v4f*>(p)); }
__device__ __forceinline__ void st4(float* p, v4f v) { __builtin_nontemporal_store(v, reinterpret_cast<v4f*>(p)); }
__device__ __forceinline__ float ld1(const float* p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ void st1(float* p, float v) { __builtin_nontemporal_store(v, p); }
// 128-bit access to an address that is only 4-byte aligned (segments of the packed buffer).
__device__ __forceinline__ v4f ld4u(const float* p) { v4f v; __builtin_memcpy(&v, p, 16); return v; }
__device__ __forceinline__ void st4u(float* p, v4f v) { __builtin_memcpy(p, &v, 16); }

// j / khw for 0 <= j < 2^22 without an integer division: a float estimate corrected by one step.
struct DivKhw {
    int khw;
    float rcp;
    __device__ __forceinline__ explicit DivKhw(int k) : khw(k), rcp(1.0f / (float)k) {}
    __device__ __forceinline__ int operator()(int j) const
    {
        if (khw == 1) return j;
        if (j >= (1 << 22)) return j / khw;
        int q = (int)((float)j * rcp);
        if (q * khw > j) --q;
        else if ((q + 1) * khw <= j) ++q;
        return q;
    }
};

__device__ __forceinline__ double wave_xor_sum(double a, int width)
{
    // butterfly over `width` adjacent lanes; every lane ends with the same bits
    for (int o = width >> 1; o > 0; o >>= 1) a += __shfl_xor(a, o, kWave);
    return a;
}

__device__ __forceinline__ int wave_sum_i32(int a)
{
    for (int o = kWave >> 1; o > 0; o >>= 1) a += __shfl_xor(a, o, kWave);
    return a;
}

__device__ __forceinline__ long long wave_sum_i64(long long a)
{
    for (int o = kWave >> 1; o > 0; o >>= 1) a += __shfl_xor(a, o, kWave);
    return a;
}

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
        const v4f u0 = ld4(a.U + e0), u1 = ld4(a.U + e1);
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
        const v4f u = ld4(a.U + e);
        const v4f wb = s * a.inv_R;
        const v4f v = wb + u;
        const v4f d = wb - v;
        st4(a.Z + e, v);
        st4(a.U + e, u + d);
        if (a.Wbar) st4(a.Wbar + e, wb);
        return v;
    }
    static __device__ __forceinline__ float scalar(const ProjectArgs& a, int Rrt, int64_t e)
    {
        const int RR = R > 0 ? R : Rrt;
        float s = ld1(a.W[0] + e);
#pragma unroll
        for (int r = 1; r < RR; ++r) s = s + ld1(a.W[r] + e);
        const float u = ld1(a.U + e);
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
template <int R>
__device__ __forceinline__ double pass1_row(const ProjectArgs& a, int Rrt, int64_t base, int row_len, bool vec,
                                            int j, int step)
{
    double acc = 0.0;
    if (vec) {
        const int nchunk = row_len >> 2;
        int c = j;
        for (; c + step < nchunk; c += 2 * step)
            acc = Cand<R>::two(a, Rrt, base + ((int64_t)c << 2), base + ((int64_t)(c + step) << 2), acc);
        if (c < nchunk) acc = sq4(acc, Cand<R>::one(a, Rrt, base + ((int64_t)c << 2)));
    } else {
        for (int c = j; c < row_len; c += step) {
            const float v = Cand<R>::scalar(a, Rrt, base + c);
            acc = fma((double)v, (double)v, acc);
        }
    }
    return acc;
}

// FILTER / NONE: a group is a row.  Short rows: `lpr` <= 64 lanes share a row and a wave covers
// 64/lpr adjacent rows.  Long rows: the whole workgroup shares a row.  Per-lane sums are combined
// by a butterfly inside the wave and (long rows) in wave order through LDS, so the order of
// additions depends only on (row_len, lpr), never on where the row sits: equal groups get equal keys.
template <int R>
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
            if (active) acc = pass1_row<R>(a, Rrt, it.base + (int64_t)rr * row_len, row_len, vec, j, lpr);
            acc = wave_xor_sum(acc, lpr);
            if (active && j == 0) a.key[it.g0 + rr] = acc;
        }
    } else {
        __shared__ double wsum[kWaves];
        for (int rr = 0; rr < it.nr; ++rr) {
            double acc = pass1_row<R>(a, Rrt, it.base + (int64_t)rr * row_len, row_len, vec, threadIdx.x, kBlock);
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
        for (int rr = wave; rr < it.nr; rr += kWaves) {
            const int64_t e = it.base + (int64_t)rr * row_len + col;
            if (vec) {
                const v4f v = Cand<R>::one(a, Rrt, e);
                acc0 = fma((double)v.x, (double)v.x, acc0);
                acc1 = fma((double)v.y, (double)v.y, acc1);
                acc2 = fma((double)v.z, (double)v.z, acc2);
                acc3 = fma((double)v.w, (double)v.w, acc3);
            } else {
                const float v = Cand<R>::scalar(a, Rrt, e);
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
    if (item_mode(it) == HSADMM_MODE_CHANNEL) project_tile<R>(it, a, Rrt);
    else project_rows<R>(it, a, Rrt);
}

// ------------------------------------------------------------------ project under a frozen mask

// Final values of 4 adjacent elements under a known mask (Algorithm 1 Phase 3, retraining branch:
// z = z~ (.) m): kept element Z = V, U += Wbar - V; masked-out element Z = +0, U = U + Wbar (= V).
template <int R>
__device__ __forceinline__ void frozen4(const ProjectArgs& a, int Rrt, int64_t e, bool k0, bool k1, bool k2, bool k3)
{
    const int RR = R > 0 ? R : Rrt;
    v4f s = ld4(a.W[0] + e);
#pragma unroll
    for (int r = 1; r < RR; ++r) s = s + ld4(a.W[r] + e);
    const v4f u = ld4(a.U + e);
    const v4f wb = s * a.inv_R;
    const v4f v = wb + u;
    v4f z;
    z.x = k0 ? v.x : 0.f; z.y = k1 ? v.y : 0.f; z.z = k2 ? v.z : 0.f; z.w = k3 ? v.w : 0.f;
    st4(a.Z + e, z);
    st4(a.U + e, u + (wb - z));
    if (a.Wbar) st4(a.Wbar + e, wb);
}

// two chunks of one row (same keep flag) with all loads issued before any store
template <int R>
__device__ __forceinline__ void frozen4x2(const ProjectArgs& a, int Rrt, int64_t e0, int64_t e1, bool keep)
{
    const int RR = R > 0 ? R : Rrt;
    v4f s0 = ld4(a.W[0] + e0), s1 = ld4(a.W[0] + e1);
#pragma unroll
    for (int r = 1; r < RR; ++r) {
        const v4f w0 = ld4(a.W[r] + e0), w1 = ld4(a.W[r] + e1);
        s0 = s0 + w0;
        s1 = s1 + w1;
    }
    const v4f u0 = ld4(a.U + e0), u1 = ld4(a.U + e1);
    const v4f wb0 = s0 * a.inv_R, wb1 = s1 * a.inv_R;
    const v4f v0 = wb0 + u0, v1 = wb1 + u1;
    const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
    const v4f z0 = keep ? v0 : zero4, z1 = keep ? v1 : zero4;
    st4(a.Z + e0, z0);
    st4(a.Z + e1, z1);
    st4(a.U + e0, u0 + (wb0 - z0));
    st4(a.U + e1, u1 + (wb1 - z1));
    if (a.Wbar) { st4(a.Wbar + e0, wb0); st4(a.Wbar + e1, wb1); }
}

template <int R>
__device__ __forceinline__ void frozen1(const ProjectArgs& a, int Rrt, int64_t e, bool keep)
{
    const int RR = R > 0 ? R : Rrt;
    float s = ld1(a.W[0] + e);
#pragma unroll
    for (int r = 1; r < RR; ++r) s = s + ld1(a.W[r] + e);
    const float u = ld1(a.U + e);
    const float wb = s * a.inv_R;
    const float v = wb + u;
    const float z = keep ? v : 0.f;
    st1(a.Z + e, z);
    st1(a.U + e, u + (wb - z));
    if (a.Wbar) st1(a.Wbar + e, wb);
}

// Same work items and lane mappings as project_pass1; no keys, no second pass: every byte of the
// replicas and of U is read once and Z and U are written once.
template <int R>
__global__ __launch_bounds__(kBlock) void project_frozen(const WorkItem* __restrict__ items, ProjectArgs a, int Rrt,
                                                         const uint8_t* __restrict__ mask)
{
    const WorkItem it = items[blockIdx.x];
    const int mode = item_mode(it);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = it.row_len;
    const bool vec = item_vec(it);
    if (mode != HSADMM_MODE_CHANNEL) {
        const int lpr = it.lpr <= kWave ? it.lpr : kBlock;
        const int rows_at_once = kBlock / lpr;
        const int sub = threadIdx.x / lpr;
        const int j = threadIdx.x - sub * lpr;
        for (int rr = sub; rr < it.nr; rr += rows_at_once) {
            const bool keep = mode == HSADMM_MODE_NONE || mask[it.g0 + rr] != 0;
            const int64_t base = it.base + (int64_t)rr * row_len;
            if (vec) {
                const int nchunk = row_len >> 2;
                int c = j;
                for (; c + lpr < nchunk; c += 2 * lpr)
                    frozen4x2<R>(a, Rrt, base + ((int64_t)c << 2), base + ((int64_t)(c + lpr) << 2), keep);
                if (c < nchunk) frozen4<R>(a, Rrt, base + ((int64_t)c << 2), keep, keep, keep, keep);
            } else {
                for (int c = j; c < row_len; c += lpr) frozen1<R>(a, Rrt, base + c, keep);
            }
        }
    } else {
        const int vw = vec ? 4 : 1;
        const int col = it.col0 + lane * vw;
        if (col >= row_len) return;
        const DivKhw div(it.khw);
        bool k[4] = {true, true, true, true};
        for (int i = 0; i < vw; ++i) k[i] = mask[it.g0 + div(col + i)] != 0;
        for (int rr = wave; rr < it.nr; rr += kWaves) {
            const int64_t e = it.base + (int64_t)rr * row_len + col;
            if (vec) frozen4<R>(a, Rrt, e, k[0], k[1], k[2], k[3]);
            else frozen1<R>(a, Rrt, e, k[0]);
        }
    }
}

// Eq. (14): out = OR of M masks, 0 / 1 bytes.
struct MaskOrArgs {
    const uint8_t* m[HSADMM_MAX_MASKS];
};

__global__ __launch_bounds__(kBlock) void mask_or_kernel(MaskOrArgs a, int M, int64_t n, uint8_t* __restrict__ out)
{
    const int64_t stride = (int64_t)gridDim.x * kBlock;
    for (int64_t g = (int64_t)blockIdx.x * kBlock + threadIdx.x; g < n; g += stride) {
        unsigned int any = 0;
        for (int i = 0; i < M; ++i) any |= a.m[i][g];
        out[g] = any != 0 ? 1 : 0;
    }
}

// ------------------------------------------------------------------ full node update (Eq. (9)) and Eq. (13)

struct WeightedArgs {
    ProjectArgs p;
    const float* Zg;      // global consensus z
    const float* Vd;      // inter-node dual v_i
    const float* coef;    // per layer: a_l, b_l
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
    u = ld4(w.p.U + e);
    const v4f q = ld4(w.Zg + e) - ld4(w.Vd + e);
    wb = s * w.p.inv_R;
    const v4f t = wb + u;
    const v4f at = t * al;
    const v4f bq = q * bl;
    zt = at + bq;
}

template <int R>
__device__ __forceinline__ void wcand1(const WeightedArgs& w, int Rrt, int64_t e, float al, float bl,
                                       float& wb, float& u, float& zt)
{
    const int RR = R > 0 ? R : Rrt;
    float s = ld1(w.p.W[0] + e);
#pragma unroll
    for (int r = 1; r < RR; ++r) s = s + ld1(w.p.W[r] + e);
    u = ld1(w.p.U + e);
    const float q = ld1(w.Zg + e) - ld1(w.Vd + e);
    wb = s * w.p.inv_R;
    const float t = wb + u;
    const float at = t * al;
    const float bq = q * bl;
    zt = at + bq;
}

// Keys of the weighted candidate: the lane mappings and the order of additions of project_pass1,
// but nothing is stored except keys / partial column sums (the selection must be known before
// anything final can be written: neither output of a group follows from the other one here).
template <int R>
__global__ __launch_bounds__(kBlock) void weighted_keys(const WorkItem* __restrict__ items, WeightedArgs w, int Rrt)
{
    __shared__ double wsum[kWaves];
    __shared__ double part[kWaves][kWave * 4];
    const WorkItem it = items[blockIdx.x];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = it.row_len;
    const bool vec = item_vec(it);
    const float al = w.coef[2 * it.layer], bl = w.coef[2 * it.layer + 1];
    if (item_mode(it) != HSADMM_MODE_CHANNEL) {
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
            if (active) {
                if (vec) {
                    const int nchunk = row_len >> 2;
                    for (int c = j; c < nchunk; c += lpr) {
                        v4f wb, u, zt;
                        wcand4<R>(w, Rrt, base + ((int64_t)c << 2), al, bl, wb, u, zt);
                        acc = sq4(acc, zt);
                    }
                } else {
                    for (int c = j; c < row_len; c += lpr) {
                        float wb, u, zt;
                        wcand1<R>(w, Rrt, base + c, al, bl, wb, u, zt);
                        acc = fma((double)zt, (double)zt, acc);
                    }
                }
            }
            if (!wide) {
                acc = wave_xor_sum(acc, lpr);
                if (active && j == 0) w.p.key[it.g0 + rr] = acc;
            } else {
                acc = wave_xor_sum(acc, kWave);
                if (lane == 0) wsum[wave] = acc;
                __syncthreads();
                if (threadIdx.x == 0) {
                    double s = wsum[0];
                    for (int v = 1; v < kWaves; ++v) s += wsum[v];
                    w.p.key[it.g0 + rr] = s;
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
                    acc0 = fma((double)zt.x, (double)zt.x, acc0);
                    acc1 = fma((double)zt.y, (double)zt.y, acc1);
                    acc2 = fma((double)zt.z, (double)zt.z, acc2);
                    acc3 = fma((double)zt.w, (double)zt.w, acc3);
                } else {
                    float wb, u, zt;
                    wcand1<R>(w, Rrt, e, al, bl, wb, u, zt);
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

// Final values once the mask is known: Z = z~ on kept groups, +0 elsewhere; U <- U + (Wbar - Z).
template <int R>
__global__ __launch_bounds__(kBlock) void weighted_final(const WorkItem* __restrict__ items, WeightedArgs w, int Rrt,
                                                         const uint8_t* __restrict__ mask)
{
    const WorkItem it = items[blockIdx.x];
    const int mode = item_mode(it);
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = it.row_len;
    const bool vec = item_vec(it);
    const float al = w.coef[2 * it.layer], bl = w.coef[2 * it.layer + 1];
    auto put4 = [&](int64_t e, bool k0, bool k1, bool k2, bool k3) {
        v4f wb, u, zt;
        wcand4<R>(w, Rrt, e, al, bl, wb, u, zt);
        v4f z;
        z.x = k0 ? zt.x : 0.f; z.y = k1 ? zt.y : 0.f; z.z = k2 ? zt.z : 0.f; z.w = k3 ? zt.w : 0.f;
        st4(w.p.Z + e, z);
        st4(w.p.U + e, u + (wb - z));
        if (w.p.Wbar) st4(w.p.Wbar + e, wb);
    };
    auto put1 = [&](int64_t e, bool keep) {
        float wb, u, zt;
        wcand1<R>(w, Rrt, e, al, bl, wb, u, zt);
        const float z = keep ? zt : 0.f;
        st1(w.p.Z + e, z);
        st1(w.p.U + e, u + (wb - z));
        if (w.p.Wbar) st1(w.p.Wbar + e, wb);
    };
    if (mode != HSADMM_MODE_CHANNEL) {
        const int lpr = it.lpr <= kWave ? it.lpr : kBlock;
        const int rows_at_once = kBlock / lpr;
        const int sub = threadIdx.x / lpr;
        const int j = threadIdx.x - sub * lpr;
        for (int rr = sub; rr < it.nr; rr += rows_at_once) {
            const bool keep = mode == HSADMM_MODE_NONE || mask[it.g0 + rr] != 0;
            const int64_t base = it.base + (int64_t)rr * row_len;
            if (vec) {
                const int nchunk = row_len >> 2;
                for (int c = j; c < nchunk; c += lpr) put4(base + ((int64_t)c << 2), keep, keep, keep, keep);
            } else {
                for (int c = j; c < row_len; c += lpr) put1(base + c, keep);
            }
        }
    } else {
        const int vw = vec ? 4 : 1;
        const int col = it.col0 + lane * vw;
        if (col >= row_len) return;
        const DivKhw div(it.khw);
        bool k[4] = {true, true, true, true};
        for (int i = 0; i < vw; ++i) k[i] = mask[it.g0 + div(col + i)] != 0;
        for (int rr = wave; rr < it.nr; rr += kWaves) {
            const int64_t e = it.base + (int64_t)rr * row_len + col;
            if (vec) put4(e, k[0], k[1], k[2], k[3]);
            else put1(e, k[0]);
        }
    }
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

// ------------------------------------------------------------------ residual norms (Algorithm 1 Phase 5)

struct ResidualArgs {
    const float* W[HSADMM_MAX_REPLICAS];
    const float* Zi;
    const float* Zi_prev;   // may be null
    const float* Zg;        // may be null
    const float* Zg_prev;   // may be null
    double* part;           // per row item: 4 partial sums
};

__device__ __forceinline__ double sqd(double acc, float a, float b)
{
    const double d = (double)a - (double)b;
    return fma(d, d, acc);
}

// One workgroup per row item (a contiguous span of one layer): per-thread fp64 sums of the four
// squared differences, combined by a butterfly per wave and in wave order through LDS.
template <int R>
__global__ __launch_bounds__(kBlock) void residual_partials(const WorkItem* __restrict__ items, ResidualArgs a, int Rrt)
{
    __shared__ double red[kWaves][4];
    const int RR = R > 0 ? R : Rrt;
    const WorkItem it = items[blockIdx.x];
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

// One workgroup per layer: adds the layer's item partials (thread t takes items t, t+256, ... in
// order; threads are combined by a butterfly per wave and in wave order), writes out[k*L + l].
__global__ __launch_bounds__(kBlock) void residual_finish(const DevLayer* __restrict__ layers, int nL,
                                                          const double* __restrict__ part, double* __restrict__ out)
{
    __shared__ double red[kWaves][4];
    const int l = blockIdx.x;
    const int first = layers[l].rows_item0, count = layers[l].rows_items;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    double s[4] = {0.0, 0.0, 0.0, 0.0};
    for (int i = threadIdx.x; i < count; i += kBlock)
        for (int k = 0; k < 4; ++k) s[k] += part[(int64_t)(first + i) * 4 + k];
    for (int k = 0; k < 4; ++k) s[k] = wave_xor_sum(s[k], kWave);
    if (lane == 0) for (int k = 0; k < 4; ++k) red[wave][k] = s[k];
    __syncthreads();
    if (threadIdx.x < 4) {
        double t = red[0][threadIdx.x];
        for (int w = 1; w < kWaves; ++w) t += red[w][threadIdx.x];
        out[(int64_t)threadIdx.x * nL + l] = t;
    }
}

// ------------------------------------------------------------------ top-k selection

// Exclusive prefix count of `flag` over the NW*64 threads of the block, in thread order.
template <int NW>
__device__ __forceinline__ int block_excl_scan(bool flag, int* wtot, int& total)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const unsigned long long b = __ballot(flag);
    const int in_wave = __popcll(b & ((1ull << lane) - 1ull));
    __syncthreads();                       // previous use of wtot is over
    if (lane == 0) wtot[wave] = __popcll(b);
    __syncthreads();
    int before = 0, tot = 0;
#pragma unroll
    for (int w = 0; w < NW; ++w) {
        const int t = wtot[w];
        before += (w < wave) ? t : 0;
        tot += t;
    }
    total = tot;
    return before + in_wave;
}

struct TopkShared {
    unsigned int hist[2][256];                 // double-buffered: one is cleared while the other fills
    unsigned long long w_and[kScanWaves], w_or[kScanWaves];
    int wtot[kScanWaves];
    unsigned long long prefix;                 // bytes of tau found so far (lower bytes zero)
    unsigned long long tau;                    // early exit: the one remaining candidate
    unsigned int need;                         // how many groups to take among the current candidates
    unsigned int cand;                         // number of current candidates
};

// Keys of a layer as seen by the selection: in registers (G <= 8 * 1024) or re-read from memory.
template <bool INREG>
struct LayerKeys {
    unsigned long long kreg[kTopkRegs];
    const unsigned long long* kb;
    int G;
    __device__ __forceinline__ void load(const unsigned long long* p, int g_count)
    {
        kb = p;
        G = g_count;
        if (INREG) {
#pragma unroll
            for (int i = 0; i < kTopkRegs; ++i) {
                const int g = (int)threadIdx.x + i * kScanBlock;
                kreg[i] = (g < G) ? kb[g] : 0ull;
            }
        }
    }
    // calls f(g, key) for every group this thread owns (g = tid, tid + 1024, ...)
    template <typename F>
    __device__ __forceinline__ void for_each(F f) const
    {
        if (INREG) {
#pragma unroll
            for (int i = 0; i < kTopkRegs; ++i) {
                const int g = (int)threadIdx.x + i * kScanBlock;
                if (g < G) f(g, kreg[i]);
            }
        } else {
            for (int g = threadIdx.x; g < G; g += kScanBlock) f(g, kb[g]);
        }
    }
};

// Keys are non-negative finite doubles, so their uint64 bit patterns order like their values.
// tau, the k-th largest pattern, is found byte by byte from the most significant byte in which the
// keys differ (one 256-bin histogram per pass).  `need` tracks how many groups must still be taken
// from the candidates that share the prefix found so far.  Groups with key > tau are kept; of the
// groups with key == tau the first `need` in index order are kept.
template <bool INREG>
__device__ __forceinline__ void topk_layer(int G, const unsigned long long* kb, uint8_t* ml, int kk, TopkShared& sh)
{
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    LayerKeys<INREG> keys;
    keys.load(kb, G);

    // bits shared by all keys
    unsigned long long a_and = ~0ull, a_or = 0ull;
    keys.for_each([&](int, unsigned long long x) { a_and &= x; a_or |= x; });
    for (int o = kWave >> 1; o > 0; o >>= 1) {
        a_and &= __shfl_xor(a_and, o, kWave);
        a_or |= __shfl_xor(a_or, o, kWave);
    }
    if (lane == 0) { sh.w_and[wave] = a_and; sh.w_or[wave] = a_or; }
    if (tid < 256) { sh.hist[0][tid] = 0u; sh.hist[1][tid] = 0u; }
    __syncthreads();
    a_and = ~0ull; a_or = 0ull;
#pragma unroll
    for (int w = 0; w < kScanWaves; ++w) { a_and &= sh.w_and[w]; a_or |= sh.w_or[w]; }
    const unsigned long long diff = a_and ^ a_or;

    unsigned long long tau;
    int need;
    bool scan_ties;
    if (diff == 0ull) {
        // all keys equal: the first k groups win
        tau = a_or;
        need = kk;
        scan_ties = true;
    } else {
        const int top = 63 - __clzll((long long)diff);        // most significant differing bit
        int shift = (top >> 3) << 3;                          // its byte
        const unsigned long long common = (shift + 8 >= 64) ? 0ull : ((a_or >> (shift + 8)) << (shift + 8));
        if (tid == 0) { sh.prefix = common; sh.need = (unsigned int)kk; sh.cand = (unsigned int)G; }
        __syncthreads();
        int buf = 0;
        bool unique = false;
        for (; shift >= 0; shift -= 8) {
            const unsigned long long prefix = sh.prefix;
            const unsigned int need_now = sh.need;
            unsigned int* h = sh.hist[buf];
            keys.for_each([&](int, unsigned long long x) {
                if (shift + 8 >= 64 || (x >> (shift + 8)) == (prefix >> (shift + 8)))
                    atomicAdd(&h[(unsigned int)(x >> shift) & 255u], 1u);
            });
            if (tid < 256) sh.hist[buf ^ 1][tid] = 0u;         // ready for the next pass
            __syncthreads();
            if (tid < kWave) {
                // lane i owns bins 4i..4i+3; `above` = number of candidates in higher bins
                const unsigned int h0 = h[4 * tid], h1 = h[4 * tid + 1], h2 = h[4 * tid + 2], h3 = h[4 * tid + 3];
                const unsigned int hh[4] = {h0, h1, h2, h3};
                const unsigned int mine = h0 + h1 + h2 + h3;
                unsigned int incl = mine;   // inclusive suffix sum over lanes tid..63
                for (int o = 1; o < kWave; o <<= 1) {
                    const unsigned int up = __shfl_down(incl, o, kWave);
                    if (tid + o < kWave) incl += up;
                }
                unsigned int above = incl - mine;
#pragma unroll
                for (int b = 3; b >= 0; --b) {
                    if (above < need_now && need_now <= above + hh[b]) {
                        sh.prefix = prefix | ((unsigned long long)(4 * tid + b) << shift);
                        sh.need = need_now - above;
                        sh.cand = hh[b];
                    }
                    above += hh[b];
                }
            }
            __syncthreads();
            buf ^= 1;
            if (sh.cand == 1u && shift > 0) { unique = true; break; }
        }
        if (unique) {
            // one candidate left: it is tau; find it by its prefix
            const unsigned long long prefix = sh.prefix;
            keys.for_each([&](int, unsigned long long x) {
                if ((x >> shift) == (prefix >> shift)) sh.tau = x;
            });
            __syncthreads();
            tau = sh.tau;
            need = 1;
            scan_ties = false;
        } else {
            tau = sh.prefix;
            need = (int)sh.need;
            scan_ties = (unsigned int)need != sh.cand;        // fewer wanted than tied: index order decides
        }
    }
    if (!scan_ties) {
        keys.for_each([&](int g, unsigned long long x) { ml[g] = (x >= tau) ? 1 : 0; });
        return;
    }
    int carry = 0;
    for (int base = 0; base < G; base += kScanBlock) {
        const int g = base + tid;
        unsigned long long x = 0ull;
        if (g < G) {
            if (INREG) {
#pragma unroll
                for (int i = 0; i < kTopkRegs; ++i) if (i * kScanBlock == base) x = keys.kreg[i];
            } else {
                x = kb[g];
            }
        }
        const bool eq = (g < G) && (x == tau);
        const bool gt = (g < G) && (x > tau);
        int total;
        const int rank = carry + block_excl_scan<kScanWaves>(eq, sh.wtot, total);
        if (g < G) ml[g] = (gt || (eq && rank < need)) ? 1 : 0;
        carry += total;
    }
}

// One workgroup per layer: finish the CHANNEL keys, then write the layer's mask.
__global__ __launch_bounds__(kScanBlock) void select_topk(const DevLayer* __restrict__ layers,
                                                          double* __restrict__ key,
                                                          const double* __restrict__ colpart,
                                                          uint8_t* __restrict__ mask)
{
    __shared__ TopkShared sh;
    const DevLayer L = layers[blockIdx.x];
    const int G = L.G;
    const int tid = threadIdx.x;
    double* kl = key + L.group_base;
    uint8_t* ml = mask + L.group_base;
    if (L.mode == HSADMM_MODE_CHANNEL) {
        // key[c] = sum over row blocks (ascending), then over the channel's khw columns (ascending)
        const double* cp = colpart + L.colpart_off;
        for (int g = tid; g < G; g += kScanBlock) {
            double acc = 0.0;
            const double* cg = cp + (int64_t)g * L.khw;
            int rb = 0;
            if (L.khw <= 9) {
                // same order of additions as the plain loop below, with four row blocks' loads in flight
                for (; rb + 4 <= L.n_rowblocks; rb += 4) {
                    double x[4][9];
#pragma unroll
                    for (int b4 = 0; b4 < 4; ++b4)
#pragma unroll
                        for (int t = 0; t < 9; ++t)
                            x[b4][t] = (t < L.khw) ? cg[(int64_t)(rb + b4) * L.row_len + t] : 0.0;
#pragma unroll
                    for (int b4 = 0; b4 < 4; ++b4)
#pragma unroll
                        for (int t = 0; t < 9; ++t)
                            if (t < L.khw) acc += x[b4][t];
                }
            }
            for (; rb < L.n_rowblocks; ++rb)
                for (int t = 0; t < L.khw; ++t) acc += cg[(int64_t)rb * L.row_len + t];
            kl[g] = acc;
        }
        __syncthreads();
    }
    const int kk = (L.mode == HSADMM_MODE_NONE) ? G : L.k;
    if (kk >= G) {
        for (int g = tid; g < G; g += kScanBlock) ml[g] = 1;
        return;
    }
    const unsigned long long* kb = reinterpret_cast<const unsigned long long*>(kl);
    if (G <= kTopkRegs * kScanBlock) topk_layer<true>(G, kb, ml, kk, sh);
    else topk_layer<false>(G, kb, ml, kk, sh);
}

// ------------------------------------------------------------------ project, fix-up of pruned groups

__global__ __launch_bounds__(kBlock) void project_fixup(const WorkItem* __restrict__ items,
                                                        const uint8_t* __restrict__ mask,
                                                        float* __restrict__ U, float* __restrict__ Z)
{
    const WorkItem it = items[blockIdx.x];
    const int mode = item_mode(it);
    if (mode == HSADMM_MODE_NONE) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = it.row_len;
    const bool vec = item_vec(it);
    const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
    if (mode == HSADMM_MODE_FILTER) {
        // lanes-per-row mapping as in pass 1 (the mapping carries no arithmetic here)
        const int lpr = it.lpr <= kWave ? it.lpr : kBlock;
        const int rows_at_once = kBlock / lpr;
        const int sub = threadIdx.x / lpr;
        const int j = threadIdx.x - sub * lpr;
        for (int rr = sub; rr < it.nr; rr += rows_at_once) {
            if (mask[it.g0 + rr]) continue;
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
    } else {
        const int vw = vec ? 4 : 1;
        const int col = it.col0 + lane * vw;
        if (col >= row_len) return;
        bool pr[4] = {false, false, false, false};
        bool any = false;
        for (int i = 0; i < vw; ++i) {
            pr[i] = mask[it.g0 + (col + i) / it.khw] == 0;
            any = any || pr[i];
        }
        if (!any) return;
        const bool all = pr[0] && pr[1] && pr[2] && pr[3];
        for (int rr = wave; rr < it.nr; rr += kWaves) {
            const int64_t e = it.base + (int64_t)rr * row_len + col;
            if (vec) {
                // a fully pruned quad moves as 128 bits; a partly pruned one stores its pruned
                // elements one by one (merging through a read of U costs more traffic than it saves)
                const v4f z = ld4(Z + e);
                if (all) {
                    st4(U + e, z);
                    st4(Z + e, zero4);
                } else {
                    if (pr[0]) { st1(U + e + 0, z.x); st1(Z + e + 0, 0.f); }
                    if (pr[1]) { st1(U + e + 1, z.y); st1(Z + e + 1, 0.f); }
                    if (pr[2]) { st1(U + e + 2, z.z); st1(Z + e + 2, 0.f); }
                    if (pr[3]) { st1(U + e + 3, z.w); st1(Z + e + 3, 0.f); }
                }
            } else {
                U[e] = Z[e];
                Z[e] = 0.f;
            }
        }
    }
}

// ------------------------------------------------------------------ mask scan (compact / expand)

struct ScanOut {
    int32_t* pos;        // groups_total: rank of a kept group inside its layer, -1 if pruned
    int32_t* cnt;        // 2L: kept groups per layer, then the start of every layer's run in kept_idx
    int64_t* layer_off;  // L+1, in the workspace (kept there for a later hsadmm_expand without a mask)
    int64_t* layer_off_out;  // L+1, the caller's copy; may be null
    int32_t* kept_idx;   // groups_total
};

__device__ __forceinline__ int nonzero_bytes(unsigned int x)
{
    // bit 7 of every byte becomes 1 iff the byte is nonzero
    const unsigned int t = (((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x) & 0x80808080u;
    return __popc(t);
}

// One workgroup per layer.  Every workgroup counts the kept groups of all layers in one flat pass
// over the mask, 16 groups per thread and step: chunk_layer gives the layer of a 16-group chunk that
// lies inside one constrained layer (one 128-bit load, a popcount, and one LDS add per wave when
// the whole wave sits in one layer); chunks that straddle layers or touch an unconstrained layer
// (0xffff) go group by group through group_layer (bit 15 marks an unconstrained layer, whose groups
// are always kept).  The workgroup then sums the aligned segment sizes of layers 0..l-1 to get its
// segment offset and scans its own layer's mask.  Segment starts are multiples of pack_align, so
// the offset is the plain sum of the rounded-up sizes.
__global__ __launch_bounds__(kScanBlock) void scan_mask(const DevLayer* __restrict__ layers, int nL,
                                                        int n_groups, int pack_align,
                                                        const uint8_t* __restrict__ mask,
                                                        const uint16_t* __restrict__ group_layer,
                                                        const uint16_t* __restrict__ chunk_layer, ScanOut o)
{
    __shared__ int cnt[HSADMM_MAX_LAYERS];
    __shared__ int wtot[kScanWaves];
    __shared__ long long wsum[kScanWaves];
    __shared__ int wkept[kScanWaves];
    const int l = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    const DevLayer L = layers[l];
    // loads that depend on nothing but the thread index go first
    long long unit_j = 0;
    int none_j = 0;
    if (tid < l) { unit_j = layers[tid].unit; none_j = layers[tid].mode == HSADMM_MODE_NONE; }
    for (int j = tid; j < nL; j += kScanBlock) cnt[j] = 0;
    __syncthreads();
    const bool aligned16 = (reinterpret_cast<uintptr_t>(mask) & 15u) == 0;
    const int nchunks = (n_groups + 15) >> 4;
    for (int c0 = wave * kWave; c0 < nchunks; c0 += kScanBlock) {
        const int c = c0 + lane;
        unsigned int cl = 0xffffu;
        int kept = 0;
        bool slow = false;
        unsigned int mw[4] = {0u, 0u, 0u, 0u};     // the chunk's 16 mask bytes
        if (c < nchunks) {
            cl = chunk_layer[c];
            const bool full = 16 * c + 15 < n_groups;
            if (full && aligned16) {
                const uint4 m = reinterpret_cast<const uint4*>(mask)[c];
                mw[0] = m.x; mw[1] = m.y; mw[2] = m.z; mw[3] = m.w;
            } else {
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    const int g = 16 * c + i;
                    const unsigned int byte = (g < n_groups) ? mask[g] : 0u;
                    mw[i >> 2] |= byte << (8 * (i & 3));
                }
            }
            if (cl != 0xffffu) kept = nonzero_bytes(mw[0]) + nonzero_bytes(mw[1]) + nonzero_bytes(mw[2]) + nonzero_bytes(mw[3]);
            else slow = true;
        }
        const unsigned int cl0 = __shfl(cl, 0, kWave);
        if (cl0 != 0xffffu && __all((c >= nchunks) || cl == cl0)) {
            const int tot = wave_sum_i32(kept);
            if (lane == 0 && tot) atomicAdd(&cnt[cl0], tot);
        } else {
            if (cl != 0xffffu && kept) atomicAdd(&cnt[cl], kept);
            if (slow) {
                // mixed chunk: the 16 layer ids come with two 128-bit loads (a partial last chunk one by one);
                // runs of one layer are counted in a register
                unsigned int gl[16];
                if (16 * c + 15 < n_groups) {
                    const uint4 a0 = reinterpret_cast<const uint4*>(group_layer)[2 * c];
                    const uint4 a1 = reinterpret_cast<const uint4*>(group_layer)[2 * c + 1];
                    const unsigned int w8[8] = {a0.x, a0.y, a0.z, a0.w, a1.x, a1.y, a1.z, a1.w};
#pragma unroll
                    for (int i = 0; i < 16; ++i) gl[i] = (w8[i >> 1] >> (16 * (i & 1))) & 0xffffu;
                } else {
#pragma unroll
                    for (int i = 0; i < 16; ++i) gl[i] = (16 * c + i < n_groups) ? group_layer[16 * c + i] : 0xffffu;
                }
                int run_layer = -1, run = 0;
#pragma unroll
                for (int i = 0; i < 16; ++i) {
                    if (gl[i] != 0xffffu) {
                        const int lay = (int)(gl[i] & 0x7fffu);
                        const unsigned int byte = (mw[i >> 2] >> (8 * (i & 3))) & 0xffu;
                        if (lay != run_layer) {
                            if (run) atomicAdd(&cnt[run_layer], run);
                            run_layer = lay;
                            run = 0;
                        }
                        run += ((gl[i] & 0x8000u) != 0 || byte != 0) ? 1 : 0;
                    }
                }
                if (run) atomicAdd(&cnt[run_layer], run);
            }
        }
    }
    __syncthreads();
    long long sz = 0;
    int kept_before = 0;
    if (tid < l) {
        const int c = cnt[tid];
        long long s = none_j ? unit_j : (long long)c * unit_j;
        sz = (s + pack_align - 1) / pack_align * pack_align;
        kept_before = c;
    }
    for (int j = tid + kScanBlock; j < l; j += kScanBlock) {    // more than 1024 layers
        const int c = cnt[j];
        long long s = (layers[j].mode == HSADMM_MODE_NONE) ? layers[j].unit : (long long)c * layers[j].unit;
        sz += (s + pack_align - 1) / pack_align * pack_align;
        kept_before += c;
    }
    sz = wave_sum_i64(sz);
    kept_before = wave_sum_i32(kept_before);
    if (lane == 0) { wsum[wave] = sz; wkept[wave] = kept_before; }
    __syncthreads();
    long long pos = 0;
    int kb = 0;
#pragma unroll
    for (int w = 0; w < kScanWaves; ++w) { pos += wsum[w]; kb += wkept[w]; }
    if (tid == 0) {
        o.layer_off[l] = pos;
        if (o.layer_off_out) o.layer_off_out[l] = pos;
        o.cnt[l] = cnt[l];
        o.cnt[nL + l] = kb;
        if (l == nL - 1) {
            long long s = (L.mode == HSADMM_MODE_NONE) ? L.unit : (long long)cnt[l] * L.unit;
            s = (s + pack_align - 1) / pack_align * pack_align;
            o.layer_off[nL] = pos + s;
            if (o.layer_off_out) o.layer_off_out[nL] = pos + s;
        }
    }
    const int G = L.G;
    int carry = 0;
    for (int base = 0; base < G; base += kScanBlock) {
        const int g = base + tid;
        const bool m = (g < G) && (L.mode == HSADMM_MODE_NONE || mask[L.group_base + g] != 0);
        int total;
        const int rank = carry + block_excl_scan<kScanWaves>(m, wtot, total);
        if (g < G) {
            o.pos[L.group_base + g] = m ? rank : -1;
            if (m) o.kept_idx[kb + rank] = g;
        }
        carry += total;
    }
}

// ------------------------------------------------------------------ compaction (gather)

// SUM: the source is the element-wise sum of two arenas (c = z_i + v_i, Section 4.4.1), formed on the fly.
template <bool SUM>
__global__ __launch_bounds__(kBlock) void compact_gather(const WorkItem* __restrict__ items,
                                                         const float* __restrict__ src,
                                                         const float* __restrict__ src1,
                                                         const int32_t* __restrict__ pos,
                                                         const int32_t* __restrict__ cnt,
                                                         const int32_t* __restrict__ kept_idx, int n_layers,
                                                         const int64_t* __restrict__ layer_off,
                                                         float* __restrict__ packed)
{
    const WorkItem it = items[blockIdx.x];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = it.row_len;
    float* out = packed + layer_off[it.layer];
    if (item_mode(it) != HSADMM_MODE_CHANNEL) {
        const int lpr = it.lpr <= kWave ? it.lpr : kBlock;
        const int rows_at_once = kBlock / lpr;
        const int sub = threadIdx.x / lpr;
        const int j = threadIdx.x - sub * lpr;
        for (int rr = sub; rr < it.nr; rr += rows_at_once) {
            const int p = pos[it.g0 + rr];
            if (p < 0) continue;
            const float* s = src + it.base + (int64_t)rr * row_len;
            const float* s1 = SUM ? src1 + it.base + (int64_t)rr * row_len : nullptr;
            float* d = out + (int64_t)p * row_len;
            if (item_vec(it)) {
                const int nchunk = row_len >> 2;
                for (int c = j; c < nchunk; c += lpr) {
                    v4f v = ld4(s + 4 * c);
                    if (SUM) v = v + ld4(s1 + 4 * c);
                    st4u(d + 4 * c, v);
                }
            } else {
                for (int c = j; c < row_len; c += lpr) d[c] = SUM ? s[c] + s1[c] : s[c];
            }
        }
    } else {
        // packed row o holds the kept channels' khw-blocks in ascending channel order: packed column
        // j = q*khw + t comes from source column kept[q]*khw + t.  it.col0 is the index of the item's
        // first row inside the layer.  A wave takes a row; a lane gathers 4 adjacent packed columns
        // and stores them with one 128-bit access.
        const int kc = cnt[it.layer];
        const int khw = it.khw;
        const int out_len = kc * khw;
        const int32_t* kl = kept_idx + cnt[n_layers + it.layer];
        const DivKhw div(khw);
        const int quads = out_len >> 2;
        for (int rr = wave; rr < it.nr; rr += kWaves) {
            const float* s = src + it.base + (int64_t)rr * row_len;
            const float* s1 = SUM ? src1 + it.base + (int64_t)rr * row_len : nullptr;
            auto at = [&](int idx) -> float { return SUM ? ld1(s + idx) + ld1(s1 + idx) : ld1(s + idx); };
            float* d = out + (int64_t)(it.col0 + rr) * out_len;
            for (int j4 = lane; j4 < quads; j4 += kWave) {
                const int j = j4 << 2;
                v4f v;
                if (khw == 1) {
                    int4 c;
                    __builtin_memcpy(&c, kl + j, 16);
                    v.x = at(c.x); v.y = at(c.y); v.z = at(c.z); v.w = at(c.w);
                } else {
                    float t4[4];
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int q = div(j + i);
                        t4[i] = at(kl[q] * khw + (j + i - q * khw));
                    }
                    v.x = t4[0]; v.y = t4[1]; v.z = t4[2]; v.w = t4[3];
                }
                st4u(d + j, v);
            }
            for (int j = (quads << 2) + lane; j < out_len; j += kWave) {
                const int q = div(j);
                d[j] = at(kl[q] * khw + (j - q * khw));
            }
        }
    }
}

// ------------------------------------------------------------------ expansion (zero fill + scatter)

__global__ __launch_bounds__(kBlock) void expand_scatter(const WorkItem* __restrict__ items,
                                                         const float* __restrict__ packed,
                                                         const int32_t* __restrict__ pos,
                                                         const int32_t* __restrict__ cnt,
                                                         const int64_t* __restrict__ layer_off,
                                                         float* __restrict__ dst)
{
    const WorkItem it = items[blockIdx.x];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = it.row_len;
    const float* in = packed + layer_off[it.layer];
    const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
    if (item_mode(it) != HSADMM_MODE_CHANNEL) {
        const int lpr = it.lpr <= kWave ? it.lpr : kBlock;
        const int rows_at_once = kBlock / lpr;
        const int sub = threadIdx.x / lpr;
        const int j = threadIdx.x - sub * lpr;
        for (int rr = sub; rr < it.nr; rr += rows_at_once) {
            const int p = pos[it.g0 + rr];
            float* d = dst + it.base + (int64_t)rr * row_len;
            const float* s = in + (int64_t)(p < 0 ? 0 : p) * row_len;
            if (item_vec(it)) {
                const int nchunk = row_len >> 2;
                if (p >= 0) for (int c = j; c < nchunk; c += lpr) st4(d + 4 * c, ld4u(s + 4 * c));
                else for (int c = j; c < nchunk; c += lpr) st4(d + 4 * c, zero4);
            } else {
                if (p >= 0) for (int c = j; c < row_len; c += lpr) d[c] = s[c];
                else for (int c = j; c < row_len; c += lpr) d[c] = 0.f;
            }
        }
    } else {
        // a wave takes a row of dst; a lane fills 4 adjacent columns (kept ones from the packed row,
        // the others +0) and stores them with one 128-bit access
        const int kc = cnt[it.layer];
        const int khw = it.khw;
        const int in_len = kc * khw;
        const DivKhw div(khw);
        const int32_t* pl = pos + it.g0;
        const int quads = item_vec(it) ? (row_len >> 2) : 0;
        for (int rr = wave; rr < it.nr; rr += kWaves) {
            float* d = dst + it.base + (int64_t)rr * row_len;
            const float* s = in + (int64_t)(it.col0 + rr) * in_len;
            for (int c4 = lane; c4 < quads; c4 += kWave) {
                const int c = c4 << 2;
                float t4[4];
                if (khw == 1) {
                    int4 p;
                    __builtin_memcpy(&p, pl + c, 16);
                    t4[0] = p.x >= 0 ? s[p.x] : 0.f;
                    t4[1] = p.y >= 0 ? s[p.y] : 0.f;
                    t4[2] = p.z >= 0 ? s[p.z] : 0.f;
                    t4[3] = p.w >= 0 ? s[p.w] : 0.f;
                } else {
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int ch = div(c + i);
                        const int p = pl[ch];
                        t4[i] = p >= 0 ? s[p * khw + (c + i - ch * khw)] : 0.f;
                    }
                }
                v4f v;
                v.x = t4[0]; v.y = t4[1]; v.z = t4[2]; v.w = t4[3];
                st4(d + c, v);
            }
            for (int c = (quads << 2) + lane; c < row_len; c += kWave) {
                const int ch = div(c);
                const int p = pl[ch];
                d[c] = (p >= 0) ? s[p * khw + (c - ch * khw)] : 0.f;
            }
        }
    }
}

// ------------------------------------------------------------------ host side

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct WsLayout {
    size_t key, colpart, pos, cnt, layer_off, kept_idx, respart, total;
};

enum KernelId { kPass1 = 0, kTopk, kFixup, kScan, kGather, kScatter, kFrozen, kMaskOr, kWKeys, kWFinal, kDualInter, kResPart, kResFinish, kKernelCount };
constexpr size_t kTimingPairs = 8192;

}  // namespace

struct hsadmm_plan {
    std::vector<hsadmm_layer_t> layers;
    std::vector<DevLayer> dev_layers;
    std::vector<WorkItem> items_proj;   // project kernels
    std::vector<WorkItem> items_rows;   // compact / expand kernels
    int32_t pack_align = 1;
    int64_t arena_elems = 0;
    int64_t groups_total = 0;
    int64_t packed_capacity = 0;
    int64_t colpart_total = 0;
    WsLayout ws{};
    int device = -1;
    DevLayer* d_layers = nullptr;
    WorkItem* d_items_proj = nullptr;
    WorkItem* d_items_rows = nullptr;
    uint16_t* d_group_layer = nullptr;   // groups_total: layer of every group (bit 15: unconstrained layer)
    float* d_coef = nullptr;             // 2L: a_l, b_l of Eq. (9), set by hsadmm_plan_set_node_weights (default 1, 0)
    uint16_t* d_chunk_layer = nullptr;   // per 16 groups: their layer if all 16 lie in one constrained layer, else 0xffff
    // Optional per-kernel timing (diagnostics; off by default).  Not thread-safe.
    bool timing = false;
    std::vector<hipEvent_t> ev;      // pairs: start, stop
    std::vector<int> ev_kernel;      // kernel id of each recorded pair
    size_t ev_used = 0;              // pairs recorded since the last read
};

namespace {

int ceil_pow2(int x)
{
    int p = 1;
    while (p < x) p *= 2;
    return p;
}

// Row items of one layer.  `mode` is the mode the kernels should see (compact / expand walk a
// CHANNEL layer row by row as well).
void add_row_items(std::vector<WorkItem>& out, int layer, const DevLayer& d, int mode)
{
    const bool vec = (d.row_len % 4) == 0;
    const int units = vec ? d.row_len / 4 : d.row_len;          // accesses per row
    int lpr, bundle;
    if (d.row_len >= kWideRow && vec) { lpr = kBlock; bundle = 1; }
    else { lpr = units >= kWave ? kWave : ceil_pow2(units); bundle = kWaves * (kWave / lpr); }
    int64_t want = kTileElems / (int64_t)d.row_len;
    if (want < bundle) want = bundle;
    want = (want + bundle - 1) / bundle * bundle;
    for (int r0 = 0; r0 < d.c_out; r0 += (int)want) {
        WorkItem it{};
        it.base = d.elem_off + (int64_t)r0 * d.row_len;
        it.aux = 0;
        it.g0 = (mode == HSADMM_MODE_CHANNEL) ? d.group_base : d.group_base + r0;
        it.nr = (int)((d.c_out - r0) < want ? (d.c_out - r0) : want);
        it.row_len = d.row_len;
        it.lpr = lpr;
        it.flags = mode | (vec ? 4 : 0);
        it.col0 = (mode == HSADMM_MODE_CHANNEL) ? r0 : 0;
        it.khw = d.khw;
        it.layer = layer;
        out.push_back(it);
    }
}

void add_tile_items(std::vector<WorkItem>& out, int layer, const DevLayer& d)
{
    const bool vec = (d.row_len % 4) == 0;
    const int strip_cols = kWave * (vec ? 4 : 1);
    const int nstrips = (d.row_len + strip_cols - 1) / strip_cols;
    for (int r0 = 0; r0 < d.c_out; r0 += kChanRows) {
        for (int s = 0; s < nstrips; ++s) {
            WorkItem it{};
            it.base = d.elem_off + (int64_t)r0 * d.row_len;
            it.aux = d.colpart_off + (int64_t)(r0 / kChanRows) * d.row_len;
            it.g0 = d.group_base;
            it.nr = (d.c_out - r0) < kChanRows ? (d.c_out - r0) : kChanRows;
            it.row_len = d.row_len;
            it.lpr = kWave;
            it.flags = HSADMM_MODE_CHANNEL | (vec ? 4 : 0);
            it.col0 = s * strip_cols;
            it.khw = d.khw;
            it.layer = layer;
            out.push_back(it);
        }
    }
}

bool is_aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// Launches `kernel` on stream s.  With timing enabled the launch carries a start and a stop event
// that take the kernel's own begin / end timestamps (no extra work is put on the stream).
template <typename... KArgs, typename... Args>
hipError_t launch(const hsadmm_plan* cp, int kid, void (*kernel)(KArgs...), unsigned grid, unsigned block,
                  hipStream_t s, Args... args)
{
    hsadmm_plan* p = const_cast<hsadmm_plan*>(cp);
    if (p->timing && p->ev_used < kTimingPairs) {
        const size_t i = p->ev_used++;
        p->ev_kernel[i] = kid;
        hipExtLaunchKernelGGL(kernel, dim3(grid), dim3(block), 0, s, p->ev[2 * i], p->ev[2 * i + 1], 0, args...);
    } else {
        hipLaunchKernelGGL(kernel, dim3(grid), dim3(block), 0, s, args...);
    }
    return hipGetLastError();
}

template <int R>
hipError_t launch_pass1(const hsadmm_plan* p, const ProjectArgs& a, int Rrt, hipStream_t s)
{
    return launch(p, kPass1, project_pass1<R>, (unsigned)p->items_proj.size(), kBlock, s,
                  (const WorkItem*)p->d_items_proj, a, Rrt);
}

template <int R>
hipError_t launch_frozen(const hsadmm_plan* p, const ProjectArgs& a, int Rrt, const uint8_t* mask, hipStream_t s)
{
    return launch(p, kFrozen, project_frozen<R>, (unsigned)p->items_proj.size(), kBlock, s,
                  (const WorkItem*)p->d_items_proj, a, Rrt, mask);
}
int run_scan(const hsadmm_plan* p, const uint8_t* mask, char* ws, int64_t* layer_off_out, int32_t* kept_idx,
             hipStream_t s)
{
    ScanOut o;
    o.pos = reinterpret_cast<int32_t*>(ws + p->ws.pos);
    o.cnt = reinterpret_cast<int32_t*>(ws + p->ws.cnt);
    o.layer_off = reinterpret_cast<int64_t*>(ws + p->ws.layer_off);
    o.layer_off_out = layer_off_out;
    o.kept_idx = kept_idx;
    const hipError_t e = launch(p, kScan, scan_mask, (unsigned)p->layers.size(), kScanBlock, s,
                                (const DevLayer*)p->d_layers, (int)p->layers.size(), (int)p->groups_total,
                                (int)p->pack_align, mask, (const uint16_t*)p->d_group_layer,
                                (const uint16_t*)p->d_chunk_layer, o);
    return e == hipSuccess ? HSADMM_OK : HSADMM_ERR_HIP;
}

}  // namespace

extern "C" {

int hsadmm_plan_create(const hsadmm_layer_t* layers, int32_t L, int32_t pack_align_elems, hsadmm_plan_t** out)
{
    if (!layers || !out || L < 1 || L > HSADMM_MAX_LAYERS || pack_align_elems < 1) return HSADMM_ERR_INVALID_ARGUMENT;
    *out = nullptr;
    int64_t prev_end = 0;
    for (int32_t l = 0; l < L; ++l) {
        const hsadmm_layer_t& x = layers[l];
        if (x.c_out < 1 || x.c_in < 1 || x.khw < 1) return HSADMM_ERR_INVALID_ARGUMENT;
        if (x.mode != HSADMM_MODE_NONE && x.mode != HSADMM_MODE_FILTER && x.mode != HSADMM_MODE_CHANNEL)
            return HSADMM_ERR_INVALID_ARGUMENT;
        const int64_t row_len = (int64_t)x.c_in * x.khw;
        const int64_t n = row_len * x.c_out;
        if (row_len > INT32_MAX || n > INT32_MAX) return HSADMM_ERR_INVALID_ARGUMENT;
        if (x.elem_off < 0 || (x.elem_off % 4) != 0 || x.elem_off < prev_end) return HSADMM_ERR_INVALID_ARGUMENT;
        const int32_t G = x.mode == HSADMM_MODE_CHANNEL ? x.c_in : x.c_out;
        if (x.mode != HSADMM_MODE_NONE && (x.k < 1 || x.k > G)) return HSADMM_ERR_INVALID_ARGUMENT;
        prev_end = x.elem_off + n;
    }
    hsadmm_plan* p = new (std::nothrow) hsadmm_plan();
    if (!p) return HSADMM_ERR_HIP;
    std::vector<uint16_t> group_layer;
    try {
        p->pack_align = pack_align_elems;
        p->layers.assign(layers, layers + L);
        p->arena_elems = prev_end;
        int64_t gb = 0, cp = 0, cap = 0;
        group_layer.clear();
        for (int32_t l = 0; l < L; ++l) {
            const hsadmm_layer_t& x = layers[l];
            DevLayer d{};
            d.elem_off = x.elem_off;
            d.c_out = x.c_out; d.c_in = x.c_in; d.khw = x.khw; d.mode = x.mode;
            d.G = x.mode == HSADMM_MODE_CHANNEL ? x.c_in : x.c_out;
            d.k = x.mode == HSADMM_MODE_NONE ? d.G : x.k;
            d.group_base = (int32_t)gb;
            d.row_len = x.c_in * x.khw;
            d.n_rowblocks = (x.c_out + kChanRows - 1) / kChanRows;
            d.colpart_off = cp;
            if (x.mode == HSADMM_MODE_CHANNEL) d.unit = (int64_t)x.c_out * x.khw;
            else if (x.mode == HSADMM_MODE_FILTER) d.unit = d.row_len;
            else d.unit = (int64_t)x.c_out * d.row_len;
            if (x.mode == HSADMM_MODE_CHANNEL) cp += (int64_t)d.n_rowblocks * d.row_len;
            gb += d.G;
            cap += (int64_t)x.c_out * d.row_len;
            cap = (cap + pack_align_elems - 1) / pack_align_elems * pack_align_elems;
            d.rows_item0 = (int32_t)p->items_rows.size();
            add_row_items(p->items_rows, l, d, x.mode);
            d.rows_items = (int32_t)p->items_rows.size() - d.rows_item0;
            if (x.mode == HSADMM_MODE_CHANNEL) add_tile_items(p->items_proj, l, d);
            else add_row_items(p->items_proj, l, d, x.mode);
            p->dev_layers.push_back(d);
            for (int32_t g = 0; g < d.G; ++g)
                group_layer.push_back((uint16_t)(l | (x.mode == HSADMM_MODE_NONE ? 0x8000 : 0)));
        }
        if (gb > INT32_MAX) { delete p; return HSADMM_ERR_UNSUPPORTED; }
        p->groups_total = gb;
        p->colpart_total = cp;
        p->packed_capacity = cap;
        size_t off = 0;
        p->ws.key = off;        off = align_up(off + sizeof(double) * (size_t)gb, 256);
        p->ws.colpart = off;    off = align_up(off + sizeof(double) * (size_t)(cp ? cp : 1), 256);
        p->ws.pos = off;        off = align_up(off + sizeof(int32_t) * (size_t)gb, 256);
        p->ws.cnt = off;        off = align_up(off + sizeof(int32_t) * (size_t)L * 2, 256);
        p->ws.layer_off = off;  off = align_up(off + sizeof(int64_t) * (size_t)(L + 1), 256);
        p->ws.kept_idx = off;   off = align_up(off + sizeof(int32_t) * (size_t)gb, 256);
        p->ws.respart = off;    off = align_up(off + sizeof(double) * 4 * p->items_rows.size(), 256);
        p->ws.total = off;
    } catch (...) {   // host allocation failure while building the tables
        delete p;
        return HSADMM_ERR_HIP;
    }

    if (hipGetDevice(&p->device) != hipSuccess) { delete p; return HSADMM_ERR_HIP; }
    const size_t bl = sizeof(DevLayer) * p->dev_layers.size();
    const size_t bp = sizeof(WorkItem) * p->items_proj.size();
    const size_t br = sizeof(WorkItem) * p->items_rows.size();
    std::vector<uint16_t> chunk_layer;
    try {
        const size_t ng = group_layer.size();
        chunk_layer.assign((ng + 15) / 16, 0xffff);
        for (size_t c = 0; c + 1 <= chunk_layer.size(); ++c) {
            if (16 * c + 15 >= ng) break;
            const uint16_t first = group_layer[16 * c];
            bool pure = (first & 0x8000) == 0;
            for (size_t i = 1; i < 16 && pure; ++i) pure = group_layer[16 * c + i] == first;
            if (pure) chunk_layer[c] = first;
        }
    } catch (...) {
        delete p;
        return HSADMM_ERR_HIP;
    }
    const size_t bg = sizeof(uint16_t) * group_layer.size();
    const size_t bc = sizeof(uint16_t) * chunk_layer.size();
    bool ok = hipMalloc(&p->d_layers, bl) == hipSuccess;
    ok = ok && hipMalloc(&p->d_items_proj, bp) == hipSuccess;
    ok = ok && hipMalloc(&p->d_items_rows, br) == hipSuccess;
    ok = ok && hipMalloc(&p->d_group_layer, bg) == hipSuccess;
    ok = ok && hipMalloc(&p->d_chunk_layer, bc) == hipSuccess;
    ok = ok && hipMalloc(&p->d_coef, sizeof(float) * 2 * p->layers.size()) == hipSuccess;
    if (ok) {
        std::vector<float> ones(2 * p->layers.size(), 0.f);
        for (size_t l = 0; l < p->layers.size(); ++l) ones[2 * l] = 1.f;
        ok = hipMemcpy(p->d_coef, ones.data(), sizeof(float) * ones.size(), hipMemcpyHostToDevice) == hipSuccess;
    }
    ok = ok && hipMemcpy(p->d_group_layer, group_layer.data(), bg, hipMemcpyHostToDevice) == hipSuccess;
    ok = ok && hipMemcpy(p->d_chunk_layer, chunk_layer.data(), bc, hipMemcpyHostToDevice) == hipSuccess;
    ok = ok && hipMemcpy(p->d_layers, p->dev_layers.data(), bl, hipMemcpyHostToDevice) == hipSuccess;
    ok = ok && hipMemcpy(p->d_items_proj, p->items_proj.data(), bp, hipMemcpyHostToDevice) == hipSuccess;
    ok = ok && hipMemcpy(p->d_items_rows, p->items_rows.data(), br, hipMemcpyHostToDevice) == hipSuccess;
    if (!ok) {
        (void)hipGetLastError();
        hsadmm_plan_destroy(p);
        return HSADMM_ERR_HIP;
    }
    *out = p;
    return HSADMM_OK;
}

void hsadmm_plan_destroy(hsadmm_plan_t* p)
{
    if (!p) return;
    for (hipEvent_t e : p->ev) (void)hipEventDestroy(e);
    if (p->d_layers) (void)hipFree(p->d_layers);
    if (p->d_items_proj) (void)hipFree(p->d_items_proj);
    if (p->d_items_rows) (void)hipFree(p->d_items_rows);
    if (p->d_group_layer) (void)hipFree(p->d_group_layer);
    if (p->d_chunk_layer) (void)hipFree(p->d_chunk_layer);
    if (p->d_coef) (void)hipFree(p->d_coef);
    delete p;
}

int hsadmm_plan_sizes(const hsadmm_plan_t* p, int64_t* arena_elems, int64_t* groups_total,
                      int64_t* packed_capacity_elems, size_t* workspace_bytes)
{
    if (!p) return HSADMM_ERR_INVALID_ARGUMENT;
    if (arena_elems) *arena_elems = p->arena_elems;
    if (groups_total) *groups_total = p->groups_total;
    if (packed_capacity_elems) *packed_capacity_elems = p->packed_capacity;
    if (workspace_bytes) *workspace_bytes = p->ws.total;
    return HSADMM_OK;
}

int hsadmm_project(const hsadmm_plan_t* p, const float* const* W_replicas, int32_t R, float* U, float* Z,
                   float* Wbar, uint8_t* mask, double* sqnorm, void* workspace, size_t workspace_bytes,
                   void* hip_stream)
{
    if (!p || !W_replicas || !U || !Z || !mask || !workspace || R < 1) return HSADMM_ERR_INVALID_ARGUMENT;
    if (R > HSADMM_MAX_REPLICAS) return HSADMM_ERR_UNSUPPORTED;
    if (!is_aligned(U, 16) || !is_aligned(Z, 16) || (Wbar && !is_aligned(Wbar, 16)) ||
        (sqnorm && !is_aligned(sqnorm, 8)) || !is_aligned(workspace, 256))
        return HSADMM_ERR_INVALID_ARGUMENT;
    for (int r = 0; r < R; ++r)
        if (!W_replicas[r] || !is_aligned(W_replicas[r], 16)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (workspace_bytes < p->ws.total) return HSADMM_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    ProjectArgs a{};
    for (int r = 0; r < R; ++r) a.W[r] = W_replicas[r];
    a.U = U; a.Z = Z; a.Wbar = Wbar;
    a.key = sqnorm ? sqnorm : reinterpret_cast<double*>(ws + p->ws.key);
    a.colpart = reinterpret_cast<double*>(ws + p->ws.colpart);
    a.inv_R = 1.0f / (float)R;
    hipError_t e;
    switch (R) {
        case 1: e = launch_pass1<1>(p, a, R, s); break;
        case 2: e = launch_pass1<2>(p, a, R, s); break;
        case 3: e = launch_pass1<3>(p, a, R, s); break;
        case 4: e = launch_pass1<4>(p, a, R, s); break;
        case 8: e = launch_pass1<8>(p, a, R, s); break;
        default: e = launch_pass1<0>(p, a, R, s); break;
    }
    if (e != hipSuccess) return HSADMM_ERR_HIP;
    e = launch(p, kTopk, select_topk, (unsigned)p->layers.size(), kScanBlock, s,
               (const DevLayer*)p->d_layers, a.key, (const double*)a.colpart, mask);
    if (e != hipSuccess) return HSADMM_ERR_HIP;
    e = launch(p, kFixup, project_fixup, (unsigned)p->items_proj.size(), kBlock, s,
               (const WorkItem*)p->d_items_proj, (const uint8_t*)mask, U, Z);
    if (e != hipSuccess) return HSADMM_ERR_HIP;
    return HSADMM_OK;
}

int hsadmm_project_frozen(const hsadmm_plan_t* p, const float* const* W_replicas, int32_t R, float* U, float* Z,
                          float* Wbar, const uint8_t* mask, void* hip_stream)
{
    if (!p || !W_replicas || !U || !Z || !mask || R < 1) return HSADMM_ERR_INVALID_ARGUMENT;
    if (R > HSADMM_MAX_REPLICAS) return HSADMM_ERR_UNSUPPORTED;
    if (!is_aligned(U, 16) || !is_aligned(Z, 16) || (Wbar && !is_aligned(Wbar, 16))) return HSADMM_ERR_INVALID_ARGUMENT;
    for (int r = 0; r < R; ++r)
        if (!W_replicas[r] || !is_aligned(W_replicas[r], 16)) return HSADMM_ERR_INVALID_ARGUMENT;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    ProjectArgs a{};
    for (int r = 0; r < R; ++r) a.W[r] = W_replicas[r];
    a.U = U; a.Z = Z; a.Wbar = Wbar;
    a.inv_R = 1.0f / (float)R;
    hipError_t e;
    switch (R) {
        case 1: e = launch_frozen<1>(p, a, R, mask, s); break;
        case 2: e = launch_frozen<2>(p, a, R, mask, s); break;
        case 3: e = launch_frozen<3>(p, a, R, mask, s); break;
        case 4: e = launch_frozen<4>(p, a, R, mask, s); break;
        case 8: e = launch_frozen<8>(p, a, R, mask, s); break;
        default: e = launch_frozen<0>(p, a, R, mask, s); break;
    }
    return e == hipSuccess ? HSADMM_OK : HSADMM_ERR_HIP;
}

int hsadmm_mask_or(const hsadmm_plan_t* p, const uint8_t* const* masks, int32_t M, uint8_t* out, void* hip_stream)
{
    if (!p || !masks || !out || M < 1) return HSADMM_ERR_INVALID_ARGUMENT;
    if (M > HSADMM_MAX_MASKS) return HSADMM_ERR_UNSUPPORTED;
    MaskOrArgs a{};
    for (int i = 0; i < M; ++i) {
        if (!masks[i]) return HSADMM_ERR_INVALID_ARGUMENT;
        a.m[i] = masks[i];
    }
    const int64_t n = p->groups_total;
    unsigned grid = (unsigned)((n + kBlock - 1) / kBlock);
    if (grid > 1024u) grid = 1024u;
    if (grid < 1u) grid = 1u;
    const hipError_t e = launch(p, kMaskOr, mask_or_kernel, grid, kBlock, static_cast<hipStream_t>(hip_stream),
                                a, (int)M, n, out);
    return e == hipSuccess ? HSADMM_OK : HSADMM_ERR_HIP;
}

static int compact_impl(const hsadmm_plan_t* p, const float* src, const float* src1, bool sum, const uint8_t* mask,
                        float* packed, int64_t* layer_off, int32_t* kept_idx, void* workspace,
                        size_t workspace_bytes, void* hip_stream)
{
    if (!p || !src || (sum && !src1) || !mask || !packed || !layer_off || !kept_idx || !workspace)
        return HSADMM_ERR_INVALID_ARGUMENT;
    if (!is_aligned(src, 16) || (sum && !is_aligned(src1, 16)) || !is_aligned(packed, 16) ||
        !is_aligned(layer_off, 8) || !is_aligned(kept_idx, 4) || !is_aligned(workspace, 256))
        return HSADMM_ERR_INVALID_ARGUMENT;
    if (workspace_bytes < p->ws.total) return HSADMM_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    const int rc = run_scan(p, mask, ws, layer_off, kept_idx, s);
    if (rc != HSADMM_OK) return rc;
    const int32_t* pos = reinterpret_cast<const int32_t*>(ws + p->ws.pos);
    const int32_t* cnt = reinterpret_cast<const int32_t*>(ws + p->ws.cnt);
    const int64_t* lo = reinterpret_cast<const int64_t*>(ws + p->ws.layer_off);
    hipError_t e;
    if (sum)
        e = launch(p, kGather, compact_gather<true>, (unsigned)p->items_rows.size(), kBlock, s,
                   (const WorkItem*)p->d_items_rows, src, src1, pos, cnt, (const int32_t*)kept_idx,
                   (int)p->layers.size(), lo, packed);
    else
        e = launch(p, kGather, compact_gather<false>, (unsigned)p->items_rows.size(), kBlock, s,
                   (const WorkItem*)p->d_items_rows, src, (const float*)nullptr, pos, cnt, (const int32_t*)kept_idx,
                   (int)p->layers.size(), lo, packed);
    return e == hipSuccess ? HSADMM_OK : HSADMM_ERR_HIP;
}

int hsadmm_compact(const hsadmm_plan_t* p, const float* src, const uint8_t* mask, float* packed,
                   int64_t* layer_off, int32_t* kept_idx, void* workspace, size_t workspace_bytes,
                   void* hip_stream)
{
    return compact_impl(p, src, nullptr, false, mask, packed, layer_off, kept_idx, workspace, workspace_bytes,
                        hip_stream);
}

int hsadmm_compact_sum(const hsadmm_plan_t* p, const float* src0, const float* src1, const uint8_t* mask,
                       float* packed, int64_t* layer_off, int32_t* kept_idx, void* workspace,
                       size_t workspace_bytes, void* hip_stream)
{
    return compact_impl(p, src0, src1, true, mask, packed, layer_off, kept_idx, workspace, workspace_bytes,
                        hip_stream);
}

int hsadmm_node_coefficients(const double* rho1, const double* rho2, int32_t L, double lambda, int32_t M, int32_t P,
                             float* a, float* b)
{
    if (!rho1 || !rho2 || !a || !b || L < 1 || M < 1 || P < 1) return HSADMM_ERR_INVALID_ARGUMENT;
    for (int32_t l = 0; l < L; ++l) {
        const double gamma = lambda / (double)M + (double)P * rho1[l] + rho2[l];
        if (!(gamma > 0.0) || rho1[l] < 0.0 || rho2[l] < 0.0) return HSADMM_ERR_INVALID_ARGUMENT;
        a[l] = (float)((double)P * rho1[l] / gamma);
        b[l] = (float)(rho2[l] / gamma);
    }
    return HSADMM_OK;
}

int hsadmm_plan_set_node_weights(hsadmm_plan_t* p, const float* a, const float* b)
{
    if (!p || !a || !b) return HSADMM_ERR_INVALID_ARGUMENT;
    const size_t L = p->layers.size();
    std::vector<float> ab;
    try {
        ab.resize(2 * L);
    } catch (...) {
        return HSADMM_ERR_HIP;
    }
    for (size_t l = 0; l < L; ++l) { ab[2 * l] = a[l]; ab[2 * l + 1] = b[l]; }
    if (hipMemcpy(p->d_coef, ab.data(), sizeof(float) * ab.size(), hipMemcpyHostToDevice) != hipSuccess)
        return HSADMM_ERR_HIP;
    return HSADMM_OK;
}

int hsadmm_project_weighted(const hsadmm_plan_t* p, const float* const* W_replicas, int32_t R, float* U,
                            const float* Zg, const float* Vd, float* Z, float* Wbar, uint8_t* mask, double* sqnorm,
                            void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!p || !W_replicas || !U || !Zg || !Vd || !Z || !mask || !workspace || R < 1) return HSADMM_ERR_INVALID_ARGUMENT;
    if (R > HSADMM_MAX_REPLICAS) return HSADMM_ERR_UNSUPPORTED;
    if (!is_aligned(U, 16) || !is_aligned(Z, 16) || !is_aligned(Zg, 16) || !is_aligned(Vd, 16) ||
        (Wbar && !is_aligned(Wbar, 16)) || (sqnorm && !is_aligned(sqnorm, 8)) || !is_aligned(workspace, 256))
        return HSADMM_ERR_INVALID_ARGUMENT;
    for (int r = 0; r < R; ++r)
        if (!W_replicas[r] || !is_aligned(W_replicas[r], 16)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (workspace_bytes < p->ws.total) return HSADMM_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    WeightedArgs w{};
    for (int r = 0; r < R; ++r) w.p.W[r] = W_replicas[r];
    w.p.U = U; w.p.Z = Z; w.p.Wbar = Wbar;
    w.p.key = sqnorm ? sqnorm : reinterpret_cast<double*>(ws + p->ws.key);
    w.p.colpart = reinterpret_cast<double*>(ws + p->ws.colpart);
    w.p.inv_R = 1.0f / (float)R;
    w.Zg = Zg; w.Vd = Vd; w.coef = p->d_coef;
    const unsigned grid = (unsigned)p->items_proj.size();
    const WorkItem* items = p->d_items_proj;
    hipError_t e;
    switch (R) {
        case 1: e = launch(p, kWKeys, weighted_keys<1>, grid, kBlock, s, items, w, (int)R); break;
        case 2: e = launch(p, kWKeys, weighted_keys<2>, grid, kBlock, s, items, w, (int)R); break;
        case 4: e = launch(p, kWKeys, weighted_keys<4>, grid, kBlock, s, items, w, (int)R); break;
        case 8: e = launch(p, kWKeys, weighted_keys<8>, grid, kBlock, s, items, w, (int)R); break;
        default: e = launch(p, kWKeys, weighted_keys<0>, grid, kBlock, s, items, w, (int)R); break;
    }
    if (e != hipSuccess) return HSADMM_ERR_HIP;
    e = launch(p, kTopk, select_topk, (unsigned)p->layers.size(), kScanBlock, s,
               (const DevLayer*)p->d_layers, w.p.key, (const double*)w.p.colpart, mask);
    if (e != hipSuccess) return HSADMM_ERR_HIP;
    const uint8_t* cm = mask;
    switch (R) {
        case 1: e = launch(p, kWFinal, weighted_final<1>, grid, kBlock, s, items, w, (int)R, cm); break;
        case 2: e = launch(p, kWFinal, weighted_final<2>, grid, kBlock, s, items, w, (int)R, cm); break;
        case 4: e = launch(p, kWFinal, weighted_final<4>, grid, kBlock, s, items, w, (int)R, cm); break;
        case 8: e = launch(p, kWFinal, weighted_final<8>, grid, kBlock, s, items, w, (int)R, cm); break;
        default: e = launch(p, kWFinal, weighted_final<0>, grid, kBlock, s, items, w, (int)R, cm); break;
    }
    return e == hipSuccess ? HSADMM_OK : HSADMM_ERR_HIP;
}

int hsadmm_residuals(const hsadmm_plan_t* p, const float* const* W_replicas, int32_t R, const float* Zi,
                     const float* Zi_prev, const float* Zg, const float* Zg_prev, double* out, void* workspace,
                     size_t workspace_bytes, void* hip_stream)
{
    if (!p || !W_replicas || !Zi || !out || !workspace || R < 1) return HSADMM_ERR_INVALID_ARGUMENT;
    if (R > HSADMM_MAX_REPLICAS) return HSADMM_ERR_UNSUPPORTED;
    if (!is_aligned(Zi, 16) || (Zi_prev && !is_aligned(Zi_prev, 16)) || (Zg && !is_aligned(Zg, 16)) ||
        (Zg_prev && !is_aligned(Zg_prev, 16)) || !is_aligned(out, 8) || !is_aligned(workspace, 256))
        return HSADMM_ERR_INVALID_ARGUMENT;
    for (int r = 0; r < R; ++r)
        if (!W_replicas[r] || !is_aligned(W_replicas[r], 16)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (workspace_bytes < p->ws.total) return HSADMM_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    ResidualArgs a{};
    for (int r = 0; r < R; ++r) a.W[r] = W_replicas[r];
    a.Zi = Zi; a.Zi_prev = Zi_prev; a.Zg = Zg; a.Zg_prev = Zg_prev;
    a.part = reinterpret_cast<double*>(static_cast<char*>(workspace) + p->ws.respart);
    const unsigned grid = (unsigned)p->items_rows.size();
    const WorkItem* items = p->d_items_rows;
    hipError_t e;
    switch (R) {
        case 1: e = launch(p, kResPart, residual_partials<1>, grid, kBlock, s, items, a, (int)R); break;
        case 2: e = launch(p, kResPart, residual_partials<2>, grid, kBlock, s, items, a, (int)R); break;
        case 4: e = launch(p, kResPart, residual_partials<4>, grid, kBlock, s, items, a, (int)R); break;
        case 8: e = launch(p, kResPart, residual_partials<8>, grid, kBlock, s, items, a, (int)R); break;
        default: e = launch(p, kResPart, residual_partials<0>, grid, kBlock, s, items, a, (int)R); break;
    }
    if (e != hipSuccess) return HSADMM_ERR_HIP;
    e = launch(p, kResFinish, residual_finish, (unsigned)p->layers.size(), kBlock, s,
               (const DevLayer*)p->d_layers, (int)p->layers.size(), (const double*)a.part, out);
    return e == hipSuccess ? HSADMM_OK : HSADMM_ERR_HIP;
}

int hsadmm_dual_inter(const hsadmm_plan_t* p, const float* Zi, const float* Zg, float* Vd, void* hip_stream)
{
    if (!p || !Zi || !Zg || !Vd) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!is_aligned(Zi, 16) || !is_aligned(Zg, 16) || !is_aligned(Vd, 16)) return HSADMM_ERR_INVALID_ARGUMENT;
    const hipError_t e = launch(p, kDualInter, dual_inter_kernel, (unsigned)p->items_rows.size(), kBlock,
                                static_cast<hipStream_t>(hip_stream), (const WorkItem*)p->d_items_rows, Zi, Zg, Vd);
    return e == hipSuccess ? HSADMM_OK : HSADMM_ERR_HIP;
}

int hsadmm_expand(const hsadmm_plan_t* p, const float* packed, const uint8_t* mask, float* dst,
                  void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!p || !packed || !dst || !workspace) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!is_aligned(packed, 16) || !is_aligned(dst, 16) || !is_aligned(workspace, 256))
        return HSADMM_ERR_INVALID_ARGUMENT;
    if (workspace_bytes < p->ws.total) return HSADMM_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    const int64_t* lo = reinterpret_cast<const int64_t*>(ws + p->ws.layer_off);
    if (mask) {
        const int rc = run_scan(p, mask, ws, nullptr, reinterpret_cast<int32_t*>(ws + p->ws.kept_idx), s);
        if (rc != HSADMM_OK) return rc;
    }   // else: the positions and offsets the last hsadmm_compact left in this workspace are used
    const hipError_t e = launch(p, kScatter, expand_scatter, (unsigned)p->items_rows.size(), kBlock, s,
                                (const WorkItem*)p->d_items_rows, packed,
                                reinterpret_cast<const int32_t*>(ws + p->ws.pos),
                                reinterpret_cast<const int32_t*>(ws + p->ws.cnt), lo, dst);
    if (e != hipSuccess) return HSADMM_ERR_HIP;
    return HSADMM_OK;
}

const char* hsadmm_strerror(int code)
{
    switch (code) {
        case HSADMM_OK: return "ok";
        case HSADMM_ERR_INVALID_ARGUMENT: return "invalid argument";
        case HSADMM_ERR_WORKSPACE: return "workspace too small";
        case HSADMM_ERR_HIP: return "HIP runtime error";
        case HSADMM_ERR_UNSUPPORTED: return "unsupported size";
        default: return "unknown error code";
    }
}

int hsadmm_version(void) { return kVersion; }

int hsadmm_kernel_timing_enable(hsadmm_plan_t* p, int enable)
{
    if (!p) return HSADMM_ERR_INVALID_ARGUMENT;
    if (enable && p->ev.empty()) {
        try {
            p->ev_kernel.assign(kTimingPairs, 0);
            p->ev.reserve(2 * kTimingPairs);
        } catch (...) {
            return HSADMM_ERR_HIP;
        }
        for (size_t i = 0; i < 2 * kTimingPairs; ++i) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) return HSADMM_ERR_HIP;
            p->ev.push_back(e);
        }
    }
    p->timing = enable != 0 && p->ev.size() == 2 * kTimingPairs;
    p->ev_used = 0;
    return HSADMM_OK;
}

int hsadmm_kernel_timing_read(hsadmm_plan_t* p, double* total_ms, int64_t* launches)
{
    if (!p || !total_ms || !launches) return HSADMM_ERR_INVALID_ARGUMENT;
    for (int k = 0; k < kKernelCount; ++k) { total_ms[k] = 0.0; launches[k] = 0; }
    for (size_t i = 0; i < p->ev_used; ++i) {
        if (hipEventSynchronize(p->ev[2 * i + 1]) != hipSuccess) return HSADMM_ERR_HIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, p->ev[2 * i], p->ev[2 * i + 1]) != hipSuccess) return HSADMM_ERR_HIP;
        total_ms[p->ev_kernel[i]] += (double)ms;
        launches[p->ev_kernel[i]] += 1;
    }
    p->ev_used = 0;
    return HSADMM_OK;
}

const char* hsadmm_kernel_name(int kernel_id)
{
    switch (kernel_id) {
        case kPass1: return "project_pass1";
        case kTopk: return "select_topk";
        case kFixup: return "project_fixup";
        case kScan: return "scan_mask";
        case kGather: return "compact_gather";
        case kScatter: return "expand_scatter";
        case kFrozen: return "project_frozen";
        case kMaskOr: return "mask_or";
        case kWKeys: return "weighted_keys";
        case kWFinal: return "weighted_final";
        case kDualInter: return "dual_inter";
        case kResPart: return "residual_partials";
        case kResFinish: return "residual_finish";
        default: return "";
    }
}

}  // extern "C"
