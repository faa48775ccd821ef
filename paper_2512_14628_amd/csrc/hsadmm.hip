// HIP kernels (gfx950 / CDNA4) and C ABI of the H-SADMM structured-sparsity step.
// The interface, data layout and arithmetic contract are stated in include/hsadmm.h.
//
// Kernel overview (every launch covers all layers of the plan through a work-item table):
//
//   project_pass1   streams the R replicas and U once.  Computes Wbar, V = Wbar + U, the fp64
//                   partial sums of V^2, and writes the values that are final if the group is
//                   kept: Z <- V, U <- U + (Wbar - V).                       [Eq. (9), (12)]
//   select_topk     one workgroup per layer: 8-pass byte-wise radix select of the k-th largest
//                   key on the uint64 view of the non-negative doubles, ties cut by an ordered
//                   scan so that lower indices win.                          [Eq. (10)]
//   project_fixup   touches pruned groups only: U <- V (taken from Z), Z <- +0.  For a pruned
//                   group U + (Wbar - 0) equals V bit for bit, so no replica is read again.
//   scan_mask       per layer: kept count, exclusive positions, kept_idx, layer_off.
//   compact_gather  packed <- src[K_out, K_in, :]                             [Eq. (15)]
//   expand_scatter  dst <- zero fill + scatter of packed                      [Section 4.4.3]
//
// Nothing here is a dense contraction, so no MFMA is used; every kernel is bound by HBM traffic.
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
constexpr int kTileElems = 8192;            // target elements per work item
constexpr int kChanRows = 64;               // CHANNEL tiles: rows per row block
constexpr int kVersion = 100;

struct DevLayer {
    int64_t elem_off;
    int64_t colpart_off;    // CHANNEL: first double of this layer's per-row-block column sums
    int32_t c_out, c_in, khw, mode, k;
    int32_t G, group_base, row_len;
    int32_t lpr;            // row-wise kernels: lanes that share one row (power of two <= 64)
    int32_t vec;            // row_len % 4 == 0 -> 128-bit accesses
    int32_t n_rowblocks;    // CHANNEL: ceil(c_out / kChanRows)
    int32_t pad_;
};

// One unit of work for a 256-thread workgroup.
//   row item  (FILTER / NONE in project kernels, every mode in compact / expand): rows [r0, r0+nr)
//   tile item (CHANNEL in project kernels): rows [r0, r0+nr) x column strip `strip`
struct WorkItem {
    int32_t layer, r0, nr, strip;
};

struct ProjectArgs {
    const float* W[HSADMM_MAX_REPLICAS];
    float* U;
    float* Z;
    float* Wbar;      // may be null
    double* key;      // groups_total
    double* colpart;  // CHANNEL partial column sums
    float inv_R;
};

__device__ __forceinline__ float4 ld4(const float* p) { return *reinterpret_cast<const float4*>(p); }
__device__ __forceinline__ void st4(float* p, float4 v) { *reinterpret_cast<float4*>(p) = v; }
// 128-bit access to an address that is only 4-byte aligned (segments of the packed buffer).
__device__ __forceinline__ float4 ld4u(const float* p) { float4 v; __builtin_memcpy(&v, p, 16); return v; }
__device__ __forceinline__ void st4u(float* p, float4 v) { __builtin_memcpy(p, &v, 16); }

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

// ------------------------------------------------------------------ project, pass 1

// Wbar, V and the dual value that is final if the group is kept, for 4 (or 1) adjacent elements.
// R > 0: replica count known at compile time (loop unrolled, pointers stay in scalar registers);
// R == 0: any replica count, taken from Rrt.
template <int R>
struct Cand {
    static __device__ __forceinline__ void v4(const ProjectArgs& a, int Rrt, int64_t e, float4& wbar, float4& v, float4& un)
    {
        const int RR = R > 0 ? R : Rrt;
        float4 s = ld4(a.W[0] + e);
#pragma unroll
        for (int r = 1; r < RR; ++r) {
            const float4 w = ld4(a.W[r] + e);
            s.x = s.x + w.x; s.y = s.y + w.y; s.z = s.z + w.z; s.w = s.w + w.w;
        }
        const float4 u = ld4(a.U + e);
        wbar.x = s.x * a.inv_R; wbar.y = s.y * a.inv_R; wbar.z = s.z * a.inv_R; wbar.w = s.w * a.inv_R;
        v.x = wbar.x + u.x; v.y = wbar.y + u.y; v.z = wbar.z + u.z; v.w = wbar.w + u.w;
        un.x = u.x + (wbar.x - v.x); un.y = u.y + (wbar.y - v.y);
        un.z = u.z + (wbar.z - v.z); un.w = u.w + (wbar.w - v.w);
    }
    static __device__ __forceinline__ void v1(const ProjectArgs& a, int Rrt, int64_t e, float& wbar, float& v, float& un)
    {
        const int RR = R > 0 ? R : Rrt;
        float s = a.W[0][e];
#pragma unroll
        for (int r = 1; r < RR; ++r) s = s + a.W[r][e];
        const float u = a.U[e];
        wbar = s * a.inv_R;
        v = wbar + u;
        un = u + (wbar - v);
    }
};

__device__ __forceinline__ double sq4(double acc, const float4& v)
{
    acc = fma((double)v.x, (double)v.x, acc);
    acc = fma((double)v.y, (double)v.y, acc);
    acc = fma((double)v.z, (double)v.z, acc);
    acc = fma((double)v.w, (double)v.w, acc);
    return acc;
}

// FILTER / NONE: a group is a row.  `lpr` lanes share a row, a wave covers 64/lpr adjacent rows,
// the waves of the workgroup take consecutive row bundles.  Lane j of a row accumulates elements
// 4j..4j+3 (+ 4*lpr*i) in order, then the lanes of the row are combined by a butterfly: the order
// of additions depends only on (row_len, lpr), never on where the row sits.
template <int R>
__device__ __forceinline__ void project_rows_impl(const DevLayer& L, const WorkItem& it, const ProjectArgs& a, int Rrt)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int lpr = L.lpr;
    const int rpw = kWave / lpr;
    const int sub = lane / lpr;
    const int j = lane - sub * lpr;
    const int row_len = L.row_len;
    for (int rb = wave * rpw; rb < it.nr; rb += kWaves * rpw) {
        const int rr = rb + sub;
        const bool active = rr < it.nr;
        const int row = it.r0 + rr;
        const int64_t base = L.elem_off + (int64_t)row * row_len;
        double acc = 0.0;
        if (active) {
            if (L.vec) {
                const int nchunk = row_len >> 2;
                for (int c = j; c < nchunk; c += lpr) {
                    const int64_t e = base + ((int64_t)c << 2);
                    float4 wbar, v, un;
                    Cand<R>::v4(a, Rrt, e, wbar, v, un);
                    st4(a.Z + e, v);
                    st4(a.U + e, un);
                    if (a.Wbar) st4(a.Wbar + e, wbar);
                    acc = sq4(acc, v);
                }
            } else {
                for (int c = j; c < row_len; c += lpr) {
                    const int64_t e = base + c;
                    float wbar, v, un;
                    Cand<R>::v1(a, Rrt, e, wbar, v, un);
                    a.Z[e] = v;
                    a.U[e] = un;
                    if (a.Wbar) a.Wbar[e] = wbar;
                    acc = fma((double)v, (double)v, acc);
                }
            }
        }
        acc = wave_xor_sum(acc, lpr);
        if (active && j == 0) a.key[L.group_base + row] = acc;
    }
}

// CHANNEL: a group is a block of khw adjacent columns of the [c_out][row_len] view.  A tile is
// (row block, column strip); each lane owns VW adjacent columns of the strip and walks down the
// rows of its wave, so it accumulates per-column sums in registers.  The four waves' sums are
// added in wave order through LDS and stored as this row block's partial column sums; select_topk
// later adds row blocks and the khw columns of a channel in a fixed order.
template <int R>
__device__ __forceinline__ void project_tile_impl(const DevLayer& L, const WorkItem& it, const ProjectArgs& a, int Rrt)
{
    __shared__ double part[kWaves][kWave * 4];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = L.row_len;
    const int vw = L.vec ? 4 : 1;
    const int col = (it.strip * kWave + lane) * vw;
    const bool in = col < row_len;
    double acc0 = 0.0, acc1 = 0.0, acc2 = 0.0, acc3 = 0.0;
    if (in) {
        for (int rr = wave; rr < it.nr; rr += kWaves) {
            const int64_t e = L.elem_off + (int64_t)(it.r0 + rr) * row_len + col;
            if (L.vec) {
                float4 wbar, v, un;
                Cand<R>::v4(a, Rrt, e, wbar, v, un);
                st4(a.Z + e, v);
                st4(a.U + e, un);
                if (a.Wbar) st4(a.Wbar + e, wbar);
                acc0 = fma((double)v.x, (double)v.x, acc0);
                acc1 = fma((double)v.y, (double)v.y, acc1);
                acc2 = fma((double)v.z, (double)v.z, acc2);
                acc3 = fma((double)v.w, (double)v.w, acc3);
            } else {
                float wbar, v, un;
                Cand<R>::v1(a, Rrt, e, wbar, v, un);
                a.Z[e] = v;
                a.U[e] = un;
                if (a.Wbar) a.Wbar[e] = wbar;
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
        const int rbi = it.r0 / kChanRows;
        double* out = a.colpart + L.colpart_off + (int64_t)rbi * row_len + col;
        for (int i = 0; i < vw; ++i) {
            double s = part[0][lane * 4 + i];
            for (int w = 1; w < kWaves; ++w) s += part[w][lane * 4 + i];
            out[i] = s;
        }
    }
}

template <int R>
__global__ __launch_bounds__(kBlock) void project_pass1(const DevLayer* __restrict__ layers,
                                                        const WorkItem* __restrict__ items,
                                                        ProjectArgs a, int Rrt)
{
    const WorkItem it = items[blockIdx.x];
    const DevLayer L = layers[it.layer];
    if (L.mode == HSADMM_MODE_CHANNEL) project_tile_impl<R>(L, it, a, Rrt);
    else project_rows_impl<R>(L, it, a, Rrt);
}

// ------------------------------------------------------------------ top-k selection

__device__ __forceinline__ int block_excl_scan_1024(bool flag, int* wtot, int& total)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const unsigned long long b = __ballot(flag);
    const int in_wave = __popcll(b & ((1ull << lane) - 1ull));
    __syncthreads();                       // previous use of wtot is over
    if (lane == 0) wtot[wave] = __popcll(b);
    __syncthreads();
    int before = 0, tot = 0;
    for (int w = 0; w < kScanWaves; ++w) {
        const int t = wtot[w];
        before += (w < wave) ? t : 0;
        tot += t;
    }
    total = tot;
    return before + in_wave;
}

// One workgroup per layer.  Keys are non-negative finite doubles, so their uint64 bit patterns
// order like their values.  The k-th largest pattern tau is found byte by byte from the top
// (256-bin histogram per pass).  Groups with key > tau are kept; of the groups with key == tau
// the first `need` in index order are kept.
__global__ __launch_bounds__(kScanBlock) void select_topk(const DevLayer* __restrict__ layers,
                                                          double* __restrict__ key,
                                                          const double* __restrict__ colpart,
                                                          uint8_t* __restrict__ mask)
{
    __shared__ unsigned int hist[256];
    __shared__ int wtot[kScanWaves];
    __shared__ unsigned long long s_prefix;
    __shared__ unsigned int s_need;
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
            for (int rb = 0; rb < L.n_rowblocks; ++rb)
                for (int t = 0; t < L.khw; ++t) acc += cp[(int64_t)rb * L.row_len + g * L.khw + t];
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
    if (tid == 0) { s_prefix = 0ull; s_need = (unsigned int)kk; }
    for (int pass = 0; pass < 8; ++pass) {
        const int shift = 56 - 8 * pass;
        if (tid < 256) hist[tid] = 0u;
        __syncthreads();
        const unsigned long long prefix = s_prefix;
        const unsigned int need = s_need;
        for (int g = tid; g < G; g += kScanBlock) {
            const unsigned long long x = kb[g];
            const bool match = (pass == 0) || ((x >> (shift + 8)) == (prefix >> (shift + 8)));
            if (match) atomicAdd(&hist[(unsigned int)(x >> shift) & 255u], 1u);
        }
        __syncthreads();
        if (tid < kWave) {
            // lane i owns bins 4i..4i+3; `above` = number of matching keys in bins of higher lanes
            const unsigned int h0 = hist[4 * tid], h1 = hist[4 * tid + 1], h2 = hist[4 * tid + 2], h3 = hist[4 * tid + 3];
            const unsigned int mine = h0 + h1 + h2 + h3;
            unsigned int incl = mine;   // inclusive suffix sum over lanes tid..63
            for (int o = 1; o < kWave; o <<= 1) {
                const unsigned int up = __shfl_down(incl, o, kWave);
                if (tid + o < kWave) incl += up;
            }
            unsigned int above = incl - mine;
            const unsigned int hh[4] = {h0, h1, h2, h3};
            for (int b = 3; b >= 0; --b) {
                if (above < need && need <= above + hh[b]) {
                    s_prefix = prefix | ((unsigned long long)(4 * tid + b) << shift);
                    s_need = need - above;
                }
                above += hh[b];
            }
        }
        __syncthreads();
    }
    const unsigned long long tau = s_prefix;
    const int need = (int)s_need;
    int carry = 0;
    for (int base = 0; base < G; base += kScanBlock) {
        const int g = base + tid;
        const unsigned long long x = (g < G) ? kb[g] : 0ull;
        const bool eq = (g < G) && (x == tau);
        const bool gt = (g < G) && (x > tau);
        int total;
        const int rank = carry + block_excl_scan_1024(eq, wtot, total);
        if (g < G) ml[g] = (gt || (eq && rank < need)) ? 1 : 0;
        carry += total;
    }
}

// ------------------------------------------------------------------ project, fix-up of pruned groups

__global__ __launch_bounds__(kBlock) void project_fixup(const DevLayer* __restrict__ layers,
                                                        const WorkItem* __restrict__ items,
                                                        const uint8_t* __restrict__ mask,
                                                        float* __restrict__ U, float* __restrict__ Z)
{
    const WorkItem it = items[blockIdx.x];
    const DevLayer L = layers[it.layer];
    if (L.mode == HSADMM_MODE_NONE) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = L.row_len;
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
    if (L.mode == HSADMM_MODE_FILTER) {
        const int lpr = L.lpr;
        const int rpw = kWave / lpr;
        const int sub = lane / lpr;
        const int j = lane - sub * lpr;
        for (int rb = wave * rpw; rb < it.nr; rb += kWaves * rpw) {
            const int rr = rb + sub;
            if (rr >= it.nr) continue;
            const int row = it.r0 + rr;
            if (mask[L.group_base + row]) continue;
            const int64_t base = L.elem_off + (int64_t)row * row_len;
            if (L.vec) {
                const int nchunk = row_len >> 2;
                for (int c = j; c < nchunk; c += lpr) {
                    const int64_t e = base + ((int64_t)c << 2);
                    st4(U + e, ld4(Z + e));
                    st4(Z + e, zero4);
                }
            } else {
                for (int c = j; c < row_len; c += lpr) {
                    U[base + c] = Z[base + c];
                    Z[base + c] = 0.f;
                }
            }
        }
    } else {
        const int vw = L.vec ? 4 : 1;
        const int col = (it.strip * kWave + lane) * vw;
        if (col >= row_len) return;
        bool pr[4] = {false, false, false, false};
        bool any = false;
        for (int i = 0; i < vw; ++i) {
            pr[i] = mask[L.group_base + (col + i) / L.khw] == 0;
            any = any || pr[i];
        }
        if (!any) return;
        for (int rr = wave; rr < it.nr; rr += kWaves) {
            const int64_t e = L.elem_off + (int64_t)(it.r0 + rr) * row_len + col;
            if (L.vec) {
                const float4 z = ld4(Z + e);
                if (pr[0] && pr[1] && pr[2] && pr[3]) {
                    st4(U + e, z);
                    st4(Z + e, zero4);
                } else {
                    if (pr[0]) { U[e + 0] = z.x; Z[e + 0] = 0.f; }
                    if (pr[1]) { U[e + 1] = z.y; Z[e + 1] = 0.f; }
                    if (pr[2]) { U[e + 2] = z.z; Z[e + 2] = 0.f; }
                    if (pr[3]) { U[e + 3] = z.w; Z[e + 3] = 0.f; }
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
    int32_t* cnt;        // L: kept groups per layer
    int64_t* layer_off;  // L+1
    int32_t* kept_idx;   // groups_total
};

__device__ __forceinline__ int64_t packed_size(const DevLayer& L, int cnt)
{
    if (L.mode == HSADMM_MODE_CHANNEL) return (int64_t)L.c_out * cnt * L.khw;
    return (int64_t)cnt * L.row_len;
}

// One workgroup per layer.  Workgroup l first counts the kept groups of layers 0..l (waves share
// the layers), derives its own segment offset, then scans its own layer's mask.
__global__ __launch_bounds__(kScanBlock) void scan_mask(const DevLayer* __restrict__ layers, int nL,
                                                        int pack_align, const uint8_t* __restrict__ mask,
                                                        ScanOut o)
{
    __shared__ int cnt[HSADMM_MAX_LAYERS];
    __shared__ int wtot[kScanWaves];
    __shared__ int s_keptbase;
    const int l = blockIdx.x;
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    for (int j = wave; j <= l; j += kScanWaves) {
        const int G = layers[j].G;
        const int gb = layers[j].group_base;
        int c = 0;
        if (layers[j].mode == HSADMM_MODE_NONE) {
            c = (lane == 0) ? G : 0;
        } else {
            for (int g = lane; g < G; g += kWave) c += mask[gb + g] != 0 ? 1 : 0;
        }
        c = wave_sum_i32(c);
        if (lane == 0) cnt[j] = c;
    }
    __syncthreads();
    const DevLayer L = layers[l];
    if (tid == 0) {
        int64_t pos = 0;
        int kb = 0;
        for (int j = 0; j < l; ++j) {
            pos += packed_size(layers[j], cnt[j]);
            pos = (pos + pack_align - 1) / pack_align * pack_align;
            kb += cnt[j];
        }
        o.layer_off[l] = pos;
        o.cnt[l] = cnt[l];
        s_keptbase = kb;
        if (l == nL - 1) {
            pos += packed_size(L, cnt[l]);
            pos = (pos + pack_align - 1) / pack_align * pack_align;
            o.layer_off[nL] = pos;
        }
    }
    __syncthreads();
    const int kb = s_keptbase;
    const int G = L.G;
    int carry = 0;
    for (int base = 0; base < G; base += kScanBlock) {
        const int g = base + tid;
        const bool m = (g < G) && (L.mode == HSADMM_MODE_NONE || mask[L.group_base + g] != 0);
        int total;
        const int rank = carry + block_excl_scan_1024(m, wtot, total);
        if (g < G) {
            o.pos[L.group_base + g] = m ? rank : -1;
            if (m) o.kept_idx[kb + rank] = g;
        }
        carry += total;
    }
}

// ------------------------------------------------------------------ compaction (gather)

__global__ __launch_bounds__(kBlock) void compact_gather(const DevLayer* __restrict__ layers,
                                                         const WorkItem* __restrict__ items,
                                                         const float* __restrict__ src,
                                                         const int32_t* __restrict__ pos,
                                                         const int32_t* __restrict__ cnt,
                                                         const int64_t* __restrict__ layer_off,
                                                         float* __restrict__ packed)
{
    const WorkItem it = items[blockIdx.x];
    const DevLayer L = layers[it.layer];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = L.row_len;
    float* out = packed + layer_off[it.layer];
    if (L.mode != HSADMM_MODE_CHANNEL) {
        const int lpr = L.lpr;
        const int rpw = kWave / lpr;
        const int sub = lane / lpr;
        const int j = lane - sub * lpr;
        for (int rb = wave * rpw; rb < it.nr; rb += kWaves * rpw) {
            const int rr = rb + sub;
            if (rr >= it.nr) continue;
            const int row = it.r0 + rr;
            const int p = pos[L.group_base + row];
            if (p < 0) continue;
            const float* s = src + L.elem_off + (int64_t)row * row_len;
            float* d = out + (int64_t)p * row_len;
            if (L.vec) {
                const int nchunk = row_len >> 2;
                for (int c = j; c < nchunk; c += lpr) st4u(d + 4 * c, ld4(s + 4 * c));
            } else {
                for (int c = j; c < row_len; c += lpr) d[c] = s[c];
            }
        }
    } else {
        // packed row o holds the kept channels' khw-blocks in ascending channel order
        const int kc = cnt[it.layer];
        const int khw = L.khw;
        const int out_len = kc * khw;
        // kept channel q of this layer -> channel index: invert pos by a search-free gather:
        // walk source columns and write each kept one to its slot.
        for (int rr = wave; rr < it.nr; rr += kWaves) {
            const int row = it.r0 + rr;
            const float* s = src + L.elem_off + (int64_t)row * row_len;
            float* d = out + (int64_t)row * out_len;
            for (int c = lane; c < row_len; c += kWave) {
                const int ch = c / khw;
                const int p = pos[L.group_base + ch];
                if (p >= 0) d[p * khw + (c - ch * khw)] = s[c];
            }
        }
    }
}

// ------------------------------------------------------------------ expansion (zero fill + scatter)

__global__ __launch_bounds__(kBlock) void expand_scatter(const DevLayer* __restrict__ layers,
                                                         const WorkItem* __restrict__ items,
                                                         const float* __restrict__ packed,
                                                         const int32_t* __restrict__ pos,
                                                         const int32_t* __restrict__ cnt,
                                                         const int64_t* __restrict__ layer_off,
                                                         float* __restrict__ dst)
{
    const WorkItem it = items[blockIdx.x];
    const DevLayer L = layers[it.layer];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = L.row_len;
    const float* in = packed + layer_off[it.layer];
    const float4 zero4 = make_float4(0.f, 0.f, 0.f, 0.f);
    if (L.mode != HSADMM_MODE_CHANNEL) {
        const int lpr = L.lpr;
        const int rpw = kWave / lpr;
        const int sub = lane / lpr;
        const int j = lane - sub * lpr;
        for (int rb = wave * rpw; rb < it.nr; rb += kWaves * rpw) {
            const int rr = rb + sub;
            if (rr >= it.nr) continue;
            const int row = it.r0 + rr;
            const int p = pos[L.group_base + row];
            float* d = dst + L.elem_off + (int64_t)row * row_len;
            const float* s = in + (int64_t)(p < 0 ? 0 : p) * row_len;
            if (L.vec) {
                const int nchunk = row_len >> 2;
                if (p >= 0) for (int c = j; c < nchunk; c += lpr) st4(d + 4 * c, ld4u(s + 4 * c));
                else for (int c = j; c < nchunk; c += lpr) st4(d + 4 * c, zero4);
            } else {
                if (p >= 0) for (int c = j; c < row_len; c += lpr) d[c] = s[c];
                else for (int c = j; c < row_len; c += lpr) d[c] = 0.f;
            }
        }
    } else {
        const int kc = cnt[it.layer];
        const int khw = L.khw;
        const int in_len = kc * khw;
        for (int rr = wave; rr < it.nr; rr += kWaves) {
            const int row = it.r0 + rr;
            float* d = dst + L.elem_off + (int64_t)row * row_len;
            const float* s = in + (int64_t)row * in_len;
            for (int c = lane; c < row_len; c += kWave) {
                const int ch = c / khw;
                const int p = pos[L.group_base + ch];
                d[c] = (p >= 0) ? s[p * khw + (c - ch * khw)] : 0.f;
            }
        }
    }
}

// ------------------------------------------------------------------ host side

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct WsLayout {
    size_t key, colpart, pos, cnt, layer_off, kept_idx, total;
};

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

void add_row_items(std::vector<WorkItem>& out, int layer, const DevLayer& d)
{
    const int rpw = kWave / d.lpr;
    const int bundle = kWaves * rpw;   // rows one pass of the workgroup covers
    int64_t want = kTileElems / (int64_t)d.row_len;
    if (want < bundle) want = bundle;
    want = (want + bundle - 1) / bundle * bundle;
    for (int r0 = 0; r0 < d.c_out; r0 += (int)want) {
        const int nr = (int)((d.c_out - r0) < want ? (d.c_out - r0) : want);
        out.push_back(WorkItem{layer, r0, nr, 0});
    }
}

bool is_aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

enum KernelId { kPass1 = 0, kTopk, kFixup, kScan, kGather, kScatter, kKernelCount };
constexpr size_t kTimingPairs = 8192;

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
                  (const DevLayer*)p->d_layers, (const WorkItem*)p->d_items_proj, a, Rrt);
}

int run_scan(const hsadmm_plan* p, const uint8_t* mask, char* ws, int64_t* layer_off, int32_t* kept_idx,
             hipStream_t s)
{
    ScanOut o;
    o.pos = reinterpret_cast<int32_t*>(ws + p->ws.pos);
    o.cnt = reinterpret_cast<int32_t*>(ws + p->ws.cnt);
    o.layer_off = layer_off;
    o.kept_idx = kept_idx;
    const hipError_t e = launch(p, kScan, scan_mask, (unsigned)p->layers.size(), kScanBlock, s,
                                (const DevLayer*)p->d_layers, (int)p->layers.size(), (int)p->pack_align, mask, o);
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
    try {
    p->pack_align = pack_align_elems;
    p->layers.assign(layers, layers + L);
    p->arena_elems = prev_end;
    int64_t gb = 0, cp = 0, cap = 0;
    for (int32_t l = 0; l < L; ++l) {
        const hsadmm_layer_t& x = layers[l];
        DevLayer d{};
        d.elem_off = x.elem_off;
        d.c_out = x.c_out; d.c_in = x.c_in; d.khw = x.khw; d.mode = x.mode;
        d.G = x.mode == HSADMM_MODE_CHANNEL ? x.c_in : x.c_out;
        d.k = x.mode == HSADMM_MODE_NONE ? d.G : x.k;
        d.group_base = (int32_t)gb;
        d.row_len = x.c_in * x.khw;
        d.vec = (d.row_len % 4) == 0 ? 1 : 0;
        const int units = d.vec ? d.row_len / 4 : d.row_len;   // accesses per row
        d.lpr = units >= kWave ? kWave : ceil_pow2(units);
        d.n_rowblocks = (x.c_out + kChanRows - 1) / kChanRows;
        d.colpart_off = cp;
        if (x.mode == HSADMM_MODE_CHANNEL) cp += (int64_t)d.n_rowblocks * d.row_len;
        gb += d.G;
        cap += (int64_t)x.c_out * d.row_len;
        cap = (cap + pack_align_elems - 1) / pack_align_elems * pack_align_elems;
        p->dev_layers.push_back(d);
        add_row_items(p->items_rows, l, d);
        if (x.mode == HSADMM_MODE_CHANNEL) {
            const int strip_cols = kWave * (d.vec ? 4 : 1);
            const int nstrips = (d.row_len + strip_cols - 1) / strip_cols;
            for (int r0 = 0; r0 < x.c_out; r0 += kChanRows) {
                const int nr = (x.c_out - r0) < kChanRows ? (x.c_out - r0) : kChanRows;
                for (int s = 0; s < nstrips; ++s) p->items_proj.push_back(WorkItem{l, r0, nr, s});
            }
        } else {
            add_row_items(p->items_proj, l, d);
        }
    }
    if (gb > INT32_MAX) { delete p; return HSADMM_ERR_UNSUPPORTED; }
    p->groups_total = gb;
    p->colpart_total = cp;
    p->packed_capacity = cap;
    size_t off = 0;
    p->ws.key = off;        off = align_up(off + sizeof(double) * (size_t)gb, 256);
    p->ws.colpart = off;    off = align_up(off + sizeof(double) * (size_t)(cp ? cp : 1), 256);
    p->ws.pos = off;        off = align_up(off + sizeof(int32_t) * (size_t)gb, 256);
    p->ws.cnt = off;        off = align_up(off + sizeof(int32_t) * (size_t)L, 256);
    p->ws.layer_off = off;  off = align_up(off + sizeof(int64_t) * (size_t)(L + 1), 256);
    p->ws.kept_idx = off;   off = align_up(off + sizeof(int32_t) * (size_t)gb, 256);
    p->ws.total = off;
    } catch (...) {   // host allocation failure while building the tables
        delete p;
        return HSADMM_ERR_HIP;
    }

    if (hipGetDevice(&p->device) != hipSuccess) { delete p; return HSADMM_ERR_HIP; }
    const size_t bl = sizeof(DevLayer) * p->dev_layers.size();
    const size_t bp = sizeof(WorkItem) * p->items_proj.size();
    const size_t br = sizeof(WorkItem) * p->items_rows.size();
    bool ok = hipMalloc(&p->d_layers, bl) == hipSuccess;
    ok = ok && hipMalloc(&p->d_items_proj, bp) == hipSuccess;
    ok = ok && hipMalloc(&p->d_items_rows, br) == hipSuccess;
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
               (const DevLayer*)p->d_layers, (const WorkItem*)p->d_items_proj, (const uint8_t*)mask, U, Z);
    if (e != hipSuccess) return HSADMM_ERR_HIP;
    return HSADMM_OK;
}

int hsadmm_compact(const hsadmm_plan_t* p, const float* src, const uint8_t* mask, float* packed,
                   int64_t* layer_off, int32_t* kept_idx, void* workspace, size_t workspace_bytes,
                   void* hip_stream)
{
    if (!p || !src || !mask || !packed || !layer_off || !kept_idx || !workspace) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!is_aligned(src, 16) || !is_aligned(packed, 16) || !is_aligned(layer_off, 8) ||
        !is_aligned(kept_idx, 4) || !is_aligned(workspace, 256))
        return HSADMM_ERR_INVALID_ARGUMENT;
    if (workspace_bytes < p->ws.total) return HSADMM_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    const int rc = run_scan(p, mask, ws, layer_off, kept_idx, s);
    if (rc != HSADMM_OK) return rc;
    const hipError_t e = launch(p, kGather, compact_gather, (unsigned)p->items_rows.size(), kBlock, s,
                                (const DevLayer*)p->d_layers, (const WorkItem*)p->d_items_rows, src,
                                reinterpret_cast<const int32_t*>(ws + p->ws.pos),
                                reinterpret_cast<const int32_t*>(ws + p->ws.cnt), (const int64_t*)layer_off, packed);
    if (e != hipSuccess) return HSADMM_ERR_HIP;
    return HSADMM_OK;
}

int hsadmm_expand(const hsadmm_plan_t* p, const float* packed, const uint8_t* mask, float* dst,
                  void* workspace, size_t workspace_bytes, void* hip_stream)
{
    if (!p || !packed || !mask || !dst || !workspace) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!is_aligned(packed, 16) || !is_aligned(dst, 16) || !is_aligned(workspace, 256))
        return HSADMM_ERR_INVALID_ARGUMENT;
    if (workspace_bytes < p->ws.total) return HSADMM_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    int64_t* lo = reinterpret_cast<int64_t*>(ws + p->ws.layer_off);
    const int rc = run_scan(p, mask, ws, lo, reinterpret_cast<int32_t*>(ws + p->ws.kept_idx), s);
    if (rc != HSADMM_OK) return rc;
    const hipError_t e = launch(p, kScatter, expand_scatter, (unsigned)p->items_rows.size(), kBlock, s,
                                (const DevLayer*)p->d_layers, (const WorkItem*)p->d_items_rows, packed,
                                reinterpret_cast<const int32_t*>(ws + p->ws.pos),
                                reinterpret_cast<const int32_t*>(ws + p->ws.cnt), (const int64_t*)lo, dst);
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
        default: return "";
    }
}

}  // extern "C"
