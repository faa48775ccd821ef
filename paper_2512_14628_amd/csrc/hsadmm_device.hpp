// Constants, work-item / argument structures and device helpers shared by every kernel.
// Part of the single translation unit built from hsadmm.hip (included there, in order).
#ifndef HSADMM_DEVICE_HPP
#define HSADMM_DEVICE_HPP
#include <hip/hip_runtime.h>
#include <cstdint>
#include "hsadmm.h"

namespace {

constexpr int kWave = 64;
constexpr int kBlock = 256;                 // streaming kernels: 4 waves
constexpr int kWaves = kBlock / kWave;
constexpr int kScanBlock = 1024;            // select_topk and scan_mask
constexpr int kScanWaves = kScanBlock / kWave;
constexpr int kTileElems = 2048;                // target elements per work item
constexpr int kWideRow = 2048;                  // rows at least this long are shared by the whole workgroup
constexpr int kChanRows = 64;               // CHANNEL tiles: rows per row block
constexpr int kBothRows = 64;               // composite_colsums tiles: rows per row block
constexpr int kTopkRegs = 8;                // the selection keeps up to 8 keys per thread in registers
constexpr int kVersion = 20100;          // 2.1.0 (major * 10000 + minor * 100 + patch)

typedef float v4f __attribute__((ext_vector_type(4)));

struct DevLayer {
    int64_t elem_off;
    int64_t colpart_off;    // CHANNEL: first double of this layer's per-row-block column sums
    int64_t packed_off;     // start of the layer in the packed buffer when exactly k (and k_in) groups are kept
    int64_t unit;           // packed elements one kept group contributes (NONE: the whole layer;
                            // BOTH: khw, the layer packs K_out * K_in * khw elements)
    int32_t c_out, c_in, khw, mode, k;
    int32_t G, group_base, row_len;   // G: groups in mask / key (BOTH: c_out filters, then c_in channels)
    int32_t n_rowblocks;    // CHANNEL: ceil(c_out / kChanRows); BOTH: ceil(c_out / kBothRows)
    int32_t rows_item0;     // first of this layer's row items (compact / expand / residual kernels)
    int32_t rows_items;     // number of them
    int32_t k_in;           // BOTH: channels kept
    int32_t seg0;           // first scan segment of the layer (a BOTH layer has two: filters, channels)
    int32_t kept_start;     // start of the layer's run in kept_idx when exactly k (and k_in) groups are kept
    // Channel groups that come in runs (CHANNEL / BOTH with khw = 1): `span` >= 1 consecutive channels make one run,
    // only k_coarse runs may hold kept channels, and nest_off is where the selection keeps its notes about the runs
    // (bytes, in the workspace's region for them).  span = 0: no such limit.
    int32_t span, k_coarse;
    int64_t nest_off;
};
static_assert(sizeof(DevLayer) == 104, "DevLayer layout");

// Packed elements of a layer that keeps c0 groups (BOTH: c0 filters and c1 channels), rounded up to pack_align.
__host__ __device__ __forceinline__ long long packed_size(int mode, long long unit, int c0, int c1, int pack_align)
{
    long long s = (mode == HSADMM_MODE_NONE) ? unit : (long long)c0 * unit;
    if (mode == HSADMM_MODE_BOTH) s *= c1;          // K_out * K_in * khw
    return (s + pack_align - 1) / pack_align * pack_align;
}

// Index mappings of the compaction, kept in the workspace: written by scan_mask from a mask, or by
// select_topk for the selection it has just made (then the counts are the plan's k / k_in).
struct IndexMaps {
    int32_t* pos;        // groups_total: rank of a kept group inside its segment, -1 if pruned
    int32_t* cnt;        // 3L: kept groups of every layer's first segment, the start of every layer's
                         // run in kept_idx, kept groups of the second segment (BOTH: channels; else 0)
    int64_t* layer_off;  // L+1
    int32_t* kept_idx;   // groups_total
    int32_t* sel;        // null, or the caller's selection record: a second copy of pos, written by select_topk only
};

// Where the first work item of every layer copies the layer's part of the index mappings held in the workspace
// (the caller's layer_off / kept_idx).
struct CopyOut {
    int64_t* layer_off;
    int32_t* kept_idx;
};

// What the selection needs to list the work a predicted selection leaves behind (sel_prev null: nothing is listed).
// The list lives in the workspace: work[0] counts the listed row items (pass 1 clears it), work[kWorkHeader + i]
// is the i-th listed item's index in the plan's table of row items.  Layers reserve their stretch of the list with
// one atomic add each, so the order of the list varies from run to run; the items are independent of each other.
constexpr int kWorkHeader = 64;
struct WorkList {
    const int32_t* sel_prev;   // the previous selection's record (the prediction); null: no list is made
    int32_t* work;
    int pack;                  // a compaction follows: kept rows whose rank has moved are listed as well
    int channels;              // CHANNEL layers were written under the prediction too: a changed layer is listed whole
    int both;                  // ... and so were the layers under both constraints
    CopyOut co;                // where the selection hands the caller layer_off / kept_idx itself (nulls: it does not)
    // residual norms taken on the way by the weighted pass 1 (null: none): for FILTER and unconstrained layers the
    // selection adds up, per layer, the sums of the outcome every group got, rows 0 and 1 of res_out
    const double* rowres;
    double* res_out;
};

// What a kernel needs to pack rows as it forms them: the index mappings (in the workspace), the packed buffer
// and where the caller wants its copies of layer_off / kept_idx.
struct PackOut {
    const int32_t* pos;
    const int32_t* cnt;
    const int32_t* kept_idx;
    const int64_t* layer_off;
    float* packed;
    CopyOut co;
    int n_layers;
};

// The whole 256-thread workgroup copies layer l's kept list and packed offset to the caller's buffers.
__device__ __forceinline__ void copy_out_layer(int l, const int32_t* cnt, const int32_t* kept_idx, int n_layers,
                                               const int64_t* layer_off, CopyOut co)
{
    const int start = cnt[n_layers + l];
    const int nk = cnt[l] + cnt[2 * n_layers + l];
    for (int i = threadIdx.x; i < nk; i += kBlock) co.kept_idx[start + i] = kept_idx[start + i];
    if (threadIdx.x == 0) {
        co.layer_off[l] = layer_off[l];
        if (l == n_layers - 1) co.layer_off[n_layers] = layer_off[n_layers];
    }
}

// One unit of work for a 256-thread workgroup; it carries everything the streaming kernels need,
// so a workgroup starts with a single 64-byte scalar load.
//   row item  (FILTER / NONE / BOTH in project kernels, every mode in compact / expand): rows [r0, r0+nr)
//   tile item (CHANNEL in project kernels, BOTH in composite_colsums): rows [r0, r0+nr) x one column strip
struct WorkItem {
    int64_t base;       // arena element offset of the item's first row (column 0)
    int64_t aux;        // tile: offset (doubles) of this row block's column sums in the workspace;
                        // BOTH row item: index in mask/pos of the layer's first channel group
    int32_t g0;         // row item: index in mask/key/pos of the first row; tile: group_base
    int32_t nr;         // rows
    int32_t row_len;    // c_in * khw
    int32_t lpr;        // row item: lanes sharing a row, power of two <= 64, or 256 (whole workgroup)
    int32_t flags;      // bits 0-1: mode; bit 2: 128-bit path (row_len % 4 == 0)
    int32_t col0;       // tile: first column of the strip; row item: 0
    int32_t khw;
    int32_t layer;
    int32_t row0;       // index of the item's first row inside the layer
    int32_t k;          // row item: groups the layer keeps under the plan's own selection (NONE: all its rows)
    int64_t packed_off; // row item: start of the layer in the packed buffer under the plan's own selection
};
static_assert(sizeof(WorkItem) == 64, "WorkItem layout");

__device__ __forceinline__ int item_mode(const WorkItem& it) { return it.flags & 3; }
// modes whose packed rows hold a subset of the columns (CHANNEL, BOTH)
__device__ __forceinline__ bool mode_has_channels(int mode) { return (mode & HSADMM_MODE_CHANNEL) != 0; }
__device__ __forceinline__ bool item_vec(const WorkItem& it) { return (it.flags & 4) != 0; }

struct ProjectArgs {
    const float* W[HSADMM_MAX_REPLICAS];
    const float* Ur;  // the dual as it is read ...
    float* U;         // ... and where the updated dual goes (the same buffer unless the caller asked for another)
    float* Z;
    float* Wbar;      // may be null
    double* key;      // groups_total
    double* colpart;  // CHANNEL partial column sums
    float inv_R;
    int park_mean;    // pass 1 parks the mean of a CHANNEL layer's replicas in Z (read back by the final pass)
    // weighted candidate of Eq. (9) (null / unused in the base projection)
    const float* Zg;      // global consensus z
    const float* Vd;      // inter-node dual v_i
    const float* coef;    // per layer: a_l, b_l
    double* respart;      // per row item: 4 partial sums of squared residuals (kernels that also form the norms)
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

// How the four waves of a workgroup share an item's rows when a wave walks a row 64 lanes at a time: with four rows
// or more a wave takes whole rows; an item of one or two rows (rows of 1024 floats and more) is shared so that no
// wave idles, four or two waves per row, each taking every fourth or second group of 64 lanes' columns.
struct WaveShare {
    int row;            // the first row this wave takes
    int rows_at_once;   // rows the workgroup works on at once (the wave's next row is this many further)
    int first;          // lane 0's first column group
    int stride;         // column groups (of one per lane) from one of the wave's steps to the next
    __device__ __forceinline__ WaveShare(int nr, int wave)
    {
        const int per_row = nr == 1 ? kWaves : (nr == 2 ? kWaves / 2 : 1);    // waves per row
        rows_at_once = kWaves / per_row;
        row = wave / per_row;
        first = (wave - row * per_row) * kWave;
        stride = per_row * kWave;
    }
};

__device__ __forceinline__ double wave_xor_sum(double a, int width)
{
    // butterfly over `width` adjacent lanes; every lane ends with the same bits
    for (int o = width >> 1; o > 0; o >>= 1) a += __shfl_xor(a, o, kWave);
    return a;
}

// acc + (a - b)^2 in fp64 (the terms of the squared residual norms of Section 3.4)
__device__ __forceinline__ double sqd(double acc, float a, float b)
{
    const double d = (double)a - (double)b;
    return fma(d, d, acc);
}

__device__ __forceinline__ double sqd4(double acc, const v4f& a, const v4f& b)
{
    acc = sqd(acc, a.x, b.x);
    acc = sqd(acc, a.y, b.y);
    acc = sqd(acc, a.z, b.z);
    return sqd(acc, a.w, b.w);
}

// Two per-thread fp64 sums of a workgroup -> dst[0], dst[1]: a butterfly per wave, then the waves in order.
__device__ __forceinline__ void block_sum_pair(double s0, double s1, double* __restrict__ dst)
{
    __shared__ double red[kWaves][2];
    s0 = wave_xor_sum(s0, kWave);
    s1 = wave_xor_sum(s1, kWave);
    if ((threadIdx.x & (kWave - 1)) == 0) { red[threadIdx.x / kWave][0] = s0; red[threadIdx.x / kWave][1] = s1; }
    __syncthreads();
    if (threadIdx.x < 2) {
        double t = red[0][threadIdx.x];
        for (int w = 1; w < kWaves; ++w) t += red[w][threadIdx.x];
        dst[threadIdx.x] = t;
    }
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

}  // namespace
#endif
