// HIP kernels (gfx950 / CDNA4) and C ABI of the H-SADMM structured-sparsity step.
// The interface, data layout and arithmetic contract are stated in include/hsadmm.h.
//
// Kernel overview (every launch covers all layers of the plan through a work-item table):
//
//   project_pass1   streams the R replicas and U once.  Computes Wbar, V = Wbar + U and the fp64
//                   partial sums of V^2; for FILTER / NONE layers it writes the values that are
//                   final if the group is kept: Z <- V, U <- U + (Wbar - V).   [Eq. (9), (12)]
//   select_topk     one workgroup per layer: radix select, eight bits a pass, of the k-th largest key on
//                   the uint64 view of the non-negative doubles (taken relative to the smallest upper
//                   word, so the first digit already spreads the keys; the last few candidates are
//                   ranked directly), ties cut by an ordered scan so that lower indices win; leaves
//                   the selection's index mappings in the workspace for a compaction / expansion
//                   without a mask.                                          [Eq. (10)]
//   project_fixup   touches pruned groups only: U <- V (taken from Z), Z <- +0.  For a pruned
//                   group U + (Wbar - 0) equals V bit for bit, so no replica is read again.
//   channel_final   CHANNEL layers: pass 1 only sums (and, with 3 or more replicas, parks their mean in Z);
//                   their Z and U are written here, in one streaming pass under the mask just selected
//                   (the kernel of the frozen-mask path, reading the parked mean instead of the replicas).
//   composite_colsums   layers under both constraints (pass 1 gives them their filter norms and parks the
//                   mean in Z): channel norms of V = Z + U over the kept filters, then a second select_topk
//                   for the channels, then the frozen-mask kernel on the parked mean writes Z and U
//                   (composite_final).                     [Section 3, paragraph after Eq. (10)]
//   scan_mask       index mappings from a given mask: kept counts, positions, kept_idx, layer_off.
//   compact_gather  packed <- src[K_out, K_in, :]                             [Eq. (15)]
//   fixup_gather    project_fixup and compact_gather of Z in one launch (hsadmm_project_compact): the
//                   first rewrites pruned rows only, the second reads kept rows only.
//   final_gather    without FILTER layers: the last final pass (with its packing) and the gather of the
//                   unconstrained layers' rows in one launch.
//   expand_scatter  dst <- zero fill + scatter of packed                      [Section 4.4.3]
//   project_frozen  one pass under a given mask; as project_frozen<R, true> it also packs the kept rows of
//                   FILTER layers and the rows of unconstrained layers (hsadmm_project_frozen_compact)  [Section 4.5]
//   weighted_pass1 / weighted_fixup   the candidate of Eq. (9) with its rho_2 term (CHANNEL and BOTH layers: the
//                   final pass is project_frozen in its weighted form, "weighted_final" in the timing table)
//   weighted_fixup_pack   weighted_fixup that also packs c = z~ + v of its kept rows, and the gather of the
//                   other layers' rows, in one launch (hsadmm_project_weighted_compact)   [Section 4.4.1]
//   dual_inter_kernel  Eq. (13);  residual_partials / residual_finish  Section 3.4;  mask_or_kernel  Eq. (14)
//   retrain_project / retrain_expand   project_frozen<R, true, true, true> and expand_scatter<true, true>: the
//                   retraining-phase iteration whose kernels also sum the squared residuals of Section 3.4
//                   (hsadmm_retrain_project, hsadmm_retrain_expand)
//
// Nothing here is a dense contraction, so no MFMA is used; every kernel is bound by HBM traffic.
// Arena data is touched once per kernel, so it is moved with non-temporal 128-bit accesses.
// fp32 arithmetic is compiled without contraction (-ffp-contract=off); the fp64 accumulation
// uses fma(v, v, acc), which equals mul+add because the square of an fp32 value is exact in fp64.
//
//   project_pass1_hinted / hinted_repair   the projection under a predicted selection (hsadmm_step with sel_prev):
//                   rows and, with the dual out of place, channels are written in the form the previous
//                   iteration's selection makes final; after the selection only what it got wrong is touched again
//
// Source layout: hsadmm_device.hpp (shared device code), kernels_*.hpp (one file per call family), this file
// (plan, launches, C ABI).  Everything is one translation unit.

#include <hip/hip_runtime.h>
#include <hip/hip_ext.h>

#include <cstdint>
#include <cstdlib>
#include <algorithm>
#include <atomic>
#include <cmath>
#include <cstring>
#include <new>
#include <type_traits>
#include <vector>

#include "hsadmm.h"

#include "hsadmm_device.hpp"
#include "kernels_project.hpp"
#include "kernels_select.hpp"
#include "kernels_frozen.hpp"
#include "kernels_hinted.hpp"
#include "kernels_estimate.hpp"
#include "kernels_weighted.hpp"
#include "kernels_residuals.hpp"
#include "kernels_compact.hpp"

namespace {

// ------------------------------------------------------------------ host side

// Calls f(std::integral_constant<int, C>{}) with C the compiled replica count that serves R: R itself when a
// kernel is specialised for it (1, 2, 4, 8; also 3 where WITH3), else 0, the form with a run-time loop over replicas.
template <bool WITH3, class F>
hipError_t for_replica_count(int R, F&& f)
{
    switch (R) {
        case 1: return f(std::integral_constant<int, 1>{});
        case 2: return f(std::integral_constant<int, 2>{});
        case 4: return f(std::integral_constant<int, 4>{});
        case 8: return f(std::integral_constant<int, 8>{});
        case 3:
            if constexpr (WITH3) return f(std::integral_constant<int, 3>{});
            else return f(std::integral_constant<int, 0>{});
        default: return f(std::integral_constant<int, 0>{});
    }
}

inline size_t align_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

struct WsLayout {
    size_t key, colpart, pos, cnt, layer_off, kept_idx, respart, work, rowres, pred, est_cnt, est_keys, est_thr, est_thr_tag, nest, total;
};

enum KernelId { kPass1 = 0, kTopk, kFixup, kScan, kGather, kScatter, kFrozen, kMaskOr, kWKeys, kWFinal, kDualInter, kResPart, kResFinish, kColsums, kChanFinal, kWFixup, kBothFinal, kAverage, kMaskDrift, kFixupGather, kWFixupPack, kRetrainProject, kRetrainExpand, kScaleLayers, kPass1Hinted, kHintedRepair, kSqnormPart, kResPick, kWHintedRepair, kKernelCount };
static_assert(kKernelCount == HSADMM_KERNEL_COUNT, "kernel id table");
constexpr size_t kTimingPairs = 8192;
constexpr size_t kRepairGrid = 2048;       // workgroups of the repair pass under a prediction: 8 per compute unit

// Scratch of the entry point that takes no workspace argument (hsadmm_project_compact_static): one array per
// device, held until the process ends.  In host code this name is only a handle for hipGetSymbolAddress; the
// device address is looked up once per plan (a plan belongs to one device) and kept in the plan.
constexpr size_t kStaticScratchBytes = HSADMM_STATIC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

}  // namespace

struct hsadmm_plan {
    std::vector<hsadmm_layer_t> layers;
    std::vector<DevLayer> dev_layers;
    std::vector<WorkItem> items_proj;   // project kernels
    std::vector<WorkItem> items_est;    // project_pass1_est: items_proj with every FILTER layer's first items ahead of the rest
    std::vector<WorkItem> items_rows;   // compact / expand kernels
    std::vector<WorkItem> items_fix;    // project_fixup, weighted_fixup: the row items of the FILTER layers
    std::vector<WorkItem> items_none;   // weighted_fixup_pack: the row items of the unconstrained layers
    std::vector<WorkItem> items_plain;  // hsadmm_project_compact: the row items of the FILTER and NONE layers
    std::vector<WorkItem> items_bfinal; // composite_final: the row items of the BOTH layers
    std::vector<WorkItem> items_chan;   // channel_final: the row items of the CHANNEL layers (a subset of items_rows)
    std::vector<WorkItem> items_both;   // composite_colsums: tiles of the layers under both constraints
    std::vector<int32_t> both_layers;   // their indices
    int32_t n_segments = 0;             // scan segments (one per layer, two per BOTH layer)
    int32_t pack_align = 1;
    int64_t arena_elems = 0;
    int64_t groups_total = 0;
    int64_t packed_capacity = 0;
    int64_t colpart_total = 0;
    WsLayout ws{};
    int device = -1;
    DevLayer* d_layers = nullptr;
    WorkItem* d_items_proj = nullptr;
    WorkItem* d_items_est = nullptr;
    WorkItem* d_items_rows = nullptr;
    WorkItem* d_items_fix = nullptr;
    WorkItem* d_items_none = nullptr;
    WorkItem* d_items_plain = nullptr;
    WorkItem* d_items_bfinal = nullptr;
    WorkItem* d_items_chan = nullptr;
    WorkItem* d_items_both = nullptr;
    int32_t* d_both_layers = nullptr;
    uint16_t* d_group_layer = nullptr;   // groups_total: scan segment of every group (bit 15: unconstrained layer)
    float* d_coef = nullptr;             // 2L: a_l, b_l of Eq. (9), set by hsadmm_plan_set_node_weights (default 1, 0)
    void* static_ws = nullptr;           // device address of `scratch` on the plan's device
    bool any_nested = false;             // some layer's channels come in runs (hsadmm_plan_create_nested)
    bool use_estimate = false;           // the un-predicted projection forms a prediction inside pass 1 (kernels_estimate.hpp)
    std::atomic<unsigned> est_calls{0};  // numbers those calls (the estimate's counts carry the number of their call)
    uint16_t* d_chunk_layer = nullptr;   // per 16 groups: their segment if all 16 lie in one constrained segment, else 0xffff
    // Optional per-kernel timing (diagnostics; off by default): the only state of a plan that changes after its
    // creation.  Launches from several host threads claim their event pairs through the atomic counter; enabling
    // and reading are for one thread at a time, with no launch of this plan in flight on another.
    bool timing = false;
    std::vector<hipEvent_t> ev;      // pairs: start, stop
    std::vector<int> ev_kernel;      // kernel id of each recorded pair
    std::atomic<size_t> ev_used{0};  // pairs claimed since the last read (may run past kTimingPairs: those launches go untimed)
    std::atomic<unsigned> last_grid[HSADMM_KERNEL_COUNT] = {};   // workgroups of the latest timed launch of every kernel
};

namespace {

// true when two buffers of n floats share an element
bool spans_overlap(const float* a, const float* b, int64_t n)
{
    const uintptr_t x = reinterpret_cast<uintptr_t>(a), y = reinterpret_cast<uintptr_t>(b);
    const uintptr_t bytes = (uintptr_t)n * sizeof(float);
    return x < y + bytes && y < x + bytes;
}

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
        it.aux = (mode == HSADMM_MODE_BOTH) ? (int64_t)d.group_base + d.c_out : 0;
        it.g0 = (mode == HSADMM_MODE_CHANNEL) ? d.group_base : d.group_base + r0;
        it.nr = (int)((d.c_out - r0) < want ? (d.c_out - r0) : want);
        it.row_len = d.row_len;
        it.lpr = lpr;
        it.flags = mode | (vec ? 4 : 0);
        it.col0 = 0;
        it.khw = d.khw;
        it.layer = layer;
        it.row0 = r0;
        it.k = d.k;
        it.packed_off = d.packed_off;
        out.push_back(it);
    }
}

// Tiles of (rows_per_block rows) x (one column strip); d.n_rowblocks must have been set for the same block height.
void add_tile_items(std::vector<WorkItem>& out, int layer, const DevLayer& d, int rows_per_block)
{
    const bool vec = (d.row_len % 4) == 0;
    const int strip_cols = kWave * (vec ? 4 : 1);
    const int nstrips = (d.row_len + strip_cols - 1) / strip_cols;
    for (int r0 = 0; r0 < d.c_out; r0 += rows_per_block) {
        for (int s = 0; s < nstrips; ++s) {
            WorkItem it{};
            it.base = d.elem_off + (int64_t)r0 * d.row_len;
            it.aux = d.colpart_off + (int64_t)(r0 / rows_per_block) * d.row_len;
            it.g0 = d.group_base;
            it.nr = (d.c_out - r0) < rows_per_block ? (d.c_out - r0) : rows_per_block;
            it.row_len = d.row_len;
            it.lpr = kWave;
            it.flags = HSADMM_MODE_CHANNEL | (vec ? 4 : 0);
            it.col0 = s * strip_cols;
            it.khw = d.khw;
            it.layer = layer;
            it.row0 = r0;
            it.k = d.k;
            it.packed_off = d.packed_off;
            out.push_back(it);
        }
    }
}

bool is_aligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }

// The plan's tables live on the device that was current when it was created; launches go to the current device.
bool on_plan_device(const hsadmm_plan* p)
{
    int d = -1;
    return hipGetDevice(&d) == hipSuccess && d == p->device;
}

// Launches `kernel` on stream s.  With timing enabled the launch carries a start and a stop event
// that take the kernel's own begin / end timestamps (no extra work is put on the stream).
template <typename... KArgs, typename... Args>
hipError_t launch(const hsadmm_plan* cp, int kid, void (*kernel)(KArgs...), unsigned grid, unsigned block,
                  hipStream_t s, Args... args)
{
    hsadmm_plan* p = const_cast<hsadmm_plan*>(cp);
    size_t i = kTimingPairs;
    if (p->timing) i = p->ev_used.fetch_add(1, std::memory_order_relaxed);
    if (i < kTimingPairs) {
        p->ev_kernel[i] = kid;
        p->last_grid[kid].store(grid, std::memory_order_relaxed);
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
    return launch(p, kFrozen, project_frozen<R>, (unsigned)p->items_rows.size(), kBlock, s,
                  (const WorkItem*)p->d_items_rows, a, Rrt, mask, PackOut{});
}

// The same pass with everything the mask keeps packed as it is formed.
template <int R>
hipError_t launch_frozen_pack(const hsadmm_plan* p, const ProjectArgs& a, int Rrt, const uint8_t* mask,
                              const PackOut& po, hipStream_t s)
{
    return launch(p, kFrozen, project_frozen<R, true>, (unsigned)p->items_rows.size(), kBlock, s,
                  (const WorkItem*)p->d_items_rows, a, Rrt, mask, po);
}

// Final Z / U of the CHANNEL layers under the mask just selected: the frozen-mask kernel over their row items.
// With 3 or more replicas pass 1 has parked their mean in Z and it is read from there (R = kMeanInZ).
template <int R>
hipError_t launch_channel_final(const hsadmm_plan* p, const ProjectArgs& a, int Rrt, const uint8_t* mask,
                                const PackOut* po, hipStream_t s)
{
    if (po)     // hsadmm_project_compact: the kept columns are packed as they are formed
        return launch(p, kChanFinal, project_frozen<R, true>, (unsigned)p->items_chan.size(), kBlock, s,
                      (const WorkItem*)p->d_items_chan, a, Rrt, mask, *po);
    return launch(p, kChanFinal, project_frozen<R>, (unsigned)p->items_chan.size(), kBlock, s,
                  (const WorkItem*)p->d_items_chan, a, Rrt, mask, PackOut{});
}
// Per-layer selection once the keys (FILTER, and the filters of BOTH) or the partial column sums
// (CHANNEL) are in place.  Layers under both constraints then take their second projection: channel
// norms over the kept filters from the candidate held in Z, and the selection of the channels.
hipError_t run_selection(const hsadmm_plan* p, double* key, double* colpart, const ProjectArgs& a, uint8_t* mask,
                         char* ws, hipStream_t s, int32_t* sel_out = nullptr, const WorkList& wl = WorkList{})
{
    // the selection also leaves its index mappings in the workspace, for a compaction without a mask
    IndexMaps im;
    im.pos = reinterpret_cast<int32_t*>(ws + p->ws.pos);
    im.cnt = reinterpret_cast<int32_t*>(ws + p->ws.cnt);
    im.layer_off = reinterpret_cast<int64_t*>(ws + p->ws.layer_off);
    im.kept_idx = reinterpret_cast<int32_t*>(ws + p->ws.kept_idx);
    im.sel = sel_out;
    const int nL = (int)p->layers.size();
    auto* const select = p->any_nested ? select_topk<true> : select_topk<false>;
    hipError_t e = launch(p, kTopk, select, (unsigned)p->layers.size(), kScanBlock, s,
                          (const DevLayer*)p->d_layers, key, (const double*)colpart, mask,
                          (const int32_t*)nullptr, 0, im, nL, (int)p->pack_align, wl, (const WorkItem*)p->d_items_rows,
                          reinterpret_cast<unsigned char*>(ws + p->ws.nest));
    if (e != hipSuccess || p->both_layers.empty()) return e;
    if (wl.both)    // pass 1 wrote these layers under the prediction: the candidate is read back from its outputs
        e = launch(p, kColsums, composite_colsums_hinted, (unsigned)p->items_both.size(), kBlock, s,
                   (const WorkItem*)p->d_items_both, (const DevLayer*)p->d_layers, (const float*)a.Z,
                   (const float*)a.U, a.Zg, a.Vd, a.coef, wl.sel_prev, (const uint8_t*)mask, colpart);
    else
        e = launch(p, kColsums, composite_colsums, (unsigned)p->items_both.size(), kBlock, s,
                   (const WorkItem*)p->d_items_both, (const float*)a.Z, a.Ur, a.Zg, a.Vd, a.coef,
                   (const uint8_t*)mask, colpart);
    if (e != hipSuccess) return e;
    return launch(p, kTopk, select, (unsigned)p->both_layers.size(), kScanBlock, s,
                  (const DevLayer*)p->d_layers, key, (const double*)colpart, mask,
                  (const int32_t*)p->d_both_layers, 1, im, nL, (int)p->pack_align, wl, (const WorkItem*)p->d_items_rows,
                  reinterpret_cast<unsigned char*>(ws + p->ws.nest));
}

int run_scan(const hsadmm_plan* p, const uint8_t* mask, char* ws, hipStream_t s, int32_t* sel_out = nullptr)
{
    IndexMaps o;
    o.pos = reinterpret_cast<int32_t*>(ws + p->ws.pos);
    o.cnt = reinterpret_cast<int32_t*>(ws + p->ws.cnt);
    o.layer_off = reinterpret_cast<int64_t*>(ws + p->ws.layer_off);
    o.kept_idx = reinterpret_cast<int32_t*>(ws + p->ws.kept_idx);
    o.sel = sel_out;
    const hipError_t e = launch(p, kScan, scan_mask, (unsigned)p->layers.size(), kScanBlock, s,
                                (const DevLayer*)p->d_layers, (int)p->layers.size(), (int)p->n_segments,
                                (int)p->groups_total,
                                (int)p->pack_align, mask, (const uint16_t*)p->d_group_layer,
                                (const uint16_t*)p->d_chunk_layer, o);
    return e == hipSuccess ? HSADMM_OK : HSADMM_ERR_HIP;
}

}  // namespace

extern "C" {

int hsadmm_plan_create(const hsadmm_layer_t* layers, int32_t L, int32_t pack_align_elems, hsadmm_plan_t** out)
{
    return hsadmm_plan_create_nested(layers, nullptr, L, pack_align_elems, out);
}

int hsadmm_plan_create_nested(const hsadmm_layer_t* layers, const hsadmm_nest_t* nest, int32_t L,
                              int32_t pack_align_elems, hsadmm_plan_t** out)
{
    if (!layers || !out || L < 1 || L > HSADMM_MAX_LAYERS || pack_align_elems < 1) return HSADMM_ERR_INVALID_ARGUMENT;
    *out = nullptr;
    int64_t prev_end = 0;
    for (int32_t l = 0; l < L; ++l) {
        const hsadmm_layer_t& x = layers[l];
        if (nest && nest[l].span >= 1) {
            // runs of channels: a layer whose groups are columns of its GEMM view, cut into whole runs, with room
            // in the kept runs for every kept column
            const hsadmm_nest_t& q = nest[l];
            if ((x.mode != HSADMM_MODE_CHANNEL && x.mode != HSADMM_MODE_BOTH) || x.khw != 1 || x.c_in < 1 ||
                (x.c_in % q.span) != 0 || q.k_coarse < 1 || q.k_coarse > x.c_in / q.span)
                return HSADMM_ERR_INVALID_ARGUMENT;
            const int64_t cols = x.mode == HSADMM_MODE_BOTH ? x.k_in : x.k;
            if (cols > (int64_t)q.k_coarse * q.span) return HSADMM_ERR_INVALID_ARGUMENT;
        }
        if (x.c_out < 1 || x.c_in < 1 || x.khw < 1) return HSADMM_ERR_INVALID_ARGUMENT;
        if (x.mode != HSADMM_MODE_NONE && x.mode != HSADMM_MODE_FILTER && x.mode != HSADMM_MODE_CHANNEL &&
            x.mode != HSADMM_MODE_BOTH)
            return HSADMM_ERR_INVALID_ARGUMENT;
        const int64_t row_len = (int64_t)x.c_in * x.khw;
        const int64_t n = row_len * x.c_out;
        if (row_len > INT32_MAX || n > INT32_MAX) return HSADMM_ERR_INVALID_ARGUMENT;
        if (x.elem_off < 0 || (x.elem_off % 4) != 0 || x.elem_off < prev_end) return HSADMM_ERR_INVALID_ARGUMENT;
        const int32_t G = x.mode == HSADMM_MODE_CHANNEL ? x.c_in : x.c_out;     // BOTH: k counts filters
        if (x.mode != HSADMM_MODE_NONE && (x.k < 1 || x.k > G)) return HSADMM_ERR_INVALID_ARGUMENT;
        if (x.mode == HSADMM_MODE_BOTH && (x.k_in < 1 || x.k_in > x.c_in)) return HSADMM_ERR_INVALID_ARGUMENT;
        prev_end = x.elem_off + n;
    }
    hsadmm_plan* p = new (std::nothrow) hsadmm_plan();
    if (!p) return HSADMM_ERR_HOST_MEMORY;
    // every plan numbers its estimating calls from a start of its own, far from the others', so that plans which take
    // turns on one workspace (the static scratch above all) do not take each other's published keys for their own
    static std::atomic<unsigned> plans_made{0};
    p->est_calls.store((plans_made.fetch_add(1, std::memory_order_relaxed) + 1u) * 0x9E3779B1u, std::memory_order_relaxed);
    std::vector<uint16_t> group_layer;
    try {
        p->pack_align = pack_align_elems;
        p->layers.assign(layers, layers + L);
        p->arena_elems = prev_end;
        int64_t gb = 0, cp = 0, cap = 0, poff = 0, nest_bytes = 0;
        int32_t seg = 0, kstart = 0;
        group_layer.clear();
        for (int32_t l = 0; l < L; ++l) {
            const hsadmm_layer_t& x = layers[l];
            DevLayer d{};
            d.elem_off = x.elem_off;
            d.c_out = x.c_out; d.c_in = x.c_in; d.khw = x.khw; d.mode = x.mode;
            const bool both = x.mode == HSADMM_MODE_BOTH;
            const bool has_colsums = x.mode == HSADMM_MODE_CHANNEL || both;
            d.G = x.mode == HSADMM_MODE_CHANNEL ? x.c_in : (both ? x.c_out + x.c_in : x.c_out);
            d.k = x.mode == HSADMM_MODE_NONE ? d.G : x.k;
            d.k_in = both ? x.k_in : 0;
            d.seg0 = seg;
            if (nest && nest[l].span >= 1) {
                // the selection's notes about the runs: their keys, the channels' shifted key patterns (8 bytes
                // each), the runs' ranks and kept list (4 bytes each), the runs' mask
                const int64_t runs = x.c_in / nest[l].span;
                d.span = nest[l].span;
                d.k_coarse = nest[l].k_coarse;
                d.nest_off = nest_bytes;
                p->any_nested = true;
                nest_bytes += (int64_t)align_up((size_t)(8 * runs + 8 * (int64_t)x.c_in + 8 * runs + runs), 8);
            }
            if (gb + d.G > INT32_MAX) { delete p; return HSADMM_ERR_UNSUPPORTED; }    // group indices are int32
            d.group_base = (int32_t)gb;
            d.row_len = x.c_in * x.khw;
            const int tile_rows = both ? kBothRows : kChanRows;
            d.n_rowblocks = (x.c_out + tile_rows - 1) / tile_rows;
            d.colpart_off = cp;
            if (x.mode == HSADMM_MODE_CHANNEL) d.unit = (int64_t)x.c_out * x.khw;
            else if (x.mode == HSADMM_MODE_FILTER) d.unit = d.row_len;
            else if (both) d.unit = x.khw;
            else d.unit = (int64_t)x.c_out * d.row_len;
            if (has_colsums) cp += (int64_t)d.n_rowblocks * d.row_len;
            // where the layer starts in the packed buffer / in kept_idx when the mask is the plan's own selection
            d.packed_off = poff;
            d.kept_start = kstart;
            const int32_t c0 = x.mode == HSADMM_MODE_NONE ? d.G : x.k;
            poff += packed_size(x.mode, d.unit, c0, d.k_in, pack_align_elems);
            kstart += c0 + d.k_in;
            gb += d.G;
            cap += (int64_t)x.c_out * d.row_len;
            cap = (cap + pack_align_elems - 1) / pack_align_elems * pack_align_elems;
            d.rows_item0 = (int32_t)p->items_rows.size();
            add_row_items(p->items_rows, l, d, x.mode);
            if (x.mode == HSADMM_MODE_NONE) add_row_items(p->items_none, l, d, x.mode);
            if (!has_colsums) add_row_items(p->items_plain, l, d, x.mode);
            d.rows_items = (int32_t)p->items_rows.size() - d.rows_item0;
            if (x.mode == HSADMM_MODE_CHANNEL) {
                add_tile_items(p->items_proj, l, d, kChanRows);
                add_row_items(p->items_chan, l, d, x.mode);
            } else {
                add_row_items(p->items_proj, l, d, x.mode);
                if (x.mode == HSADMM_MODE_FILTER) add_row_items(p->items_fix, l, d, x.mode);
                if (x.mode == HSADMM_MODE_BOTH) {
                    add_row_items(p->items_bfinal, l, d, x.mode);
                }
            }
            if (both) {
                add_tile_items(p->items_both, l, d, kBothRows);
                p->both_layers.push_back(l);
            }
            p->dev_layers.push_back(d);
            // scan segments: at most 2 * HSADMM_MAX_LAYERS = 8192, so an id fits below bit 15
            for (int32_t g = 0; g < d.G; ++g) {
                const int32_t sg = seg + ((both && g >= x.c_out) ? 1 : 0);
                group_layer.push_back((uint16_t)(sg | (x.mode == HSADMM_MODE_NONE ? 0x8000 : 0)));
            }
            seg += both ? 2 : 1;
        }
        p->n_segments = seg;
        p->groups_total = gb;
        p->colpart_total = cp;
        p->packed_capacity = cap;
        size_t off = 0;
        p->ws.key = off;        off = align_up(off + sizeof(double) * (size_t)gb, 256);
        p->ws.colpart = off;    off = align_up(off + sizeof(double) * (size_t)(cp ? cp : 1), 256);
        p->ws.pos = off;        off = align_up(off + sizeof(int32_t) * (size_t)gb, 256);
        p->ws.cnt = off;        off = align_up(off + sizeof(int32_t) * (size_t)L * 3, 256);
        p->ws.layer_off = off;  off = align_up(off + sizeof(int64_t) * (size_t)(L + 1), 256);
        p->ws.kept_idx = off;   off = align_up(off + sizeof(int32_t) * (size_t)gb, 256);
        p->ws.respart = off;    off = align_up(off + sizeof(double) * 4 * p->items_rows.size(), 256);
        p->ws.work = off;       off = align_up(off + sizeof(int32_t) * (kWorkHeader + p->items_rows.size()), 256);
        p->ws.rowres = off;     off = align_up(off + sizeof(double) * 4 * (size_t)gb, 256);
        p->ws.pred = off;       off = align_up(off + sizeof(int32_t) * (size_t)gb, 256);
        p->ws.est_cnt = off;    off = align_up(off + sizeof(unsigned int) * (size_t)L * kSampleKeys, 256);
        p->ws.est_keys = off;   off = align_up(off + sizeof(double) * (size_t)L * kSampleKeys, 256);
        p->ws.est_thr = off;    off = align_up(off + sizeof(double) * (size_t)L, 256);
        p->ws.est_thr_tag = off; off = align_up(off + sizeof(unsigned int) * (size_t)L, 256);
        p->ws.nest = off;       off = align_up(off + (size_t)nest_bytes, 256);
        p->ws.total = off;
        // The estimate's item order: of every FILTER layer the items that cover its first rows (a sixteenth of them,
        // 16 at least, kSampleKeys at most), then everything else in the usual order.
        bool only_rows = true, any_filter = false;
        for (int32_t l = 0; l < L; ++l) {
            only_rows = only_rows && (layers[l].mode == HSADMM_MODE_FILTER || layers[l].mode == HSADMM_MODE_NONE);
            any_filter = any_filter || layers[l].mode == HSADMM_MODE_FILTER;
        }
        // (the first rows' detour costs a few microseconds per launch whatever the size: measured a loss on plans of
        // 12 M elements and less, a gain from 25 M on)
        int64_t n_elems_total = 0;
        for (int32_t l = 0; l < L; ++l) n_elems_total += (int64_t)layers[l].c_out * layers[l].c_in * layers[l].khw;
        // (environment, read here once per plan: HSADMM_NO_ESTIMATE switches the path off, HSADMM_FORCE_ESTIMATE takes
        // it whatever the size, which is how the tests reach it with small tables)
        p->use_estimate = only_rows && any_filter && std::getenv("HSADMM_NO_ESTIMATE") == nullptr &&
                          (n_elems_total >= kEstimateMinElems || std::getenv("HSADMM_FORCE_ESTIMATE") != nullptr);
        if (p->use_estimate) {
            std::vector<WorkItem> rest;
            for (WorkItem it : p->items_proj) {
                const DevLayer& d = p->dev_layers[it.layer];
                const bool filter = (it.flags & 3) == HSADMM_MODE_FILTER;
                const bool holds = filter && (it.flags & 4) != 0 && (int64_t)it.nr * it.row_len <= kStageElems &&
                                   it.nr <= kStageRows;
                const int sample_rows = sample_rows_of(d.G);
                it.col0 = !holds ? kEstPlain : (it.row0 < sample_rows ? kEstSample : kEstUse);
                if (it.col0 == kEstSample) p->items_est.push_back(it);
                else rest.push_back(it);
            }
            p->items_est.insert(p->items_est.end(), rest.begin(), rest.end());
        }
    } catch (...) {   // host allocation failure while building the tables
        delete p;
        return HSADMM_ERR_HOST_MEMORY;
    }

    if (hipGetDevice(&p->device) != hipSuccess) { delete p; return HSADMM_ERR_HIP; }
    // this device's copy of the static scratch array (every device holds its own, at its own address)
    if (hipGetSymbolAddress(&p->static_ws, HIP_SYMBOL(scratch)) != hipSuccess || p->static_ws == nullptr) {
        (void)hipGetLastError();
        delete p;
        return HSADMM_ERR_HIP;
    }
    std::vector<uint16_t> chunk_layer;
    std::vector<float> coef;
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
        coef.assign(2 * p->layers.size(), 0.f);                  // a_l = 1, b_l = 0
        for (size_t l = 0; l < p->layers.size(); ++l) coef[2 * l] = 1.f;
    } catch (...) {
        delete p;
        return HSADMM_ERR_HOST_MEMORY;
    }
    // device copies of the tables (an empty table stays a null pointer and is never launched over)
    bool ok = true;
    auto upload = [&ok](const auto& v, auto** d) {
        if (v.empty() || !ok) return;
        const size_t bytes = sizeof(v[0]) * v.size();
        ok = hipMalloc(reinterpret_cast<void**>(d), bytes) == hipSuccess &&
             hipMemcpy(*d, v.data(), bytes, hipMemcpyHostToDevice) == hipSuccess;
    };
    upload(p->dev_layers, &p->d_layers);
    upload(p->items_proj, &p->d_items_proj);
    upload(p->items_rows, &p->d_items_rows);
    upload(p->items_fix, &p->d_items_fix);
    upload(p->items_none, &p->d_items_none);
    upload(p->items_est, &p->d_items_est);
    upload(p->items_plain, &p->d_items_plain);
    upload(p->items_bfinal, &p->d_items_bfinal);
    upload(p->items_chan, &p->d_items_chan);
    upload(p->items_both, &p->d_items_both);
    upload(p->both_layers, &p->d_both_layers);
    upload(group_layer, &p->d_group_layer);
    upload(chunk_layer, &p->d_chunk_layer);
    upload(coef, &p->d_coef);
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
    if (p->d_items_fix) (void)hipFree(p->d_items_fix);
    if (p->d_items_none) (void)hipFree(p->d_items_none);
    if (p->d_items_est) (void)hipFree(p->d_items_est);
    if (p->d_items_plain) (void)hipFree(p->d_items_plain);
    if (p->d_items_bfinal) (void)hipFree(p->d_items_bfinal);
    if (p->d_items_chan) (void)hipFree(p->d_items_chan);
    if (p->d_items_both) (void)hipFree(p->d_items_both);
    if (p->d_both_layers) (void)hipFree(p->d_both_layers);
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

// Where hsadmm_project_compact sends the compaction of Z (all NULL: no compaction).
struct CompactOut {
    float* packed;
    int64_t* layer_off;
    int32_t* kept_idx;
};

// sel_prev: the previous selection's record, which predicts this one (null: no prediction); sel_out: receives this
// selection's record (may be null).
static int project_impl(const hsadmm_plan_t* p, const float* const* W_replicas, int32_t R, float* U, float* Z,
                        float* Wbar, uint8_t* mask, double* sqnorm, const CompactOut* out, void* workspace,
                        size_t workspace_bytes, void* hip_stream, const int32_t* sel_prev = nullptr,
                        int32_t* sel_out = nullptr, float* U_out = nullptr)
{
    if (!p || !W_replicas || !U || !Z || !mask || !workspace || R < 1) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!is_aligned(sel_prev, 4) || !is_aligned(sel_out, 4) || !is_aligned(U_out, 16)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (U_out && (spans_overlap(U_out, U, p->arena_elems) || spans_overlap(U_out, Z, p->arena_elems)))
        return HSADMM_ERR_INVALID_ARGUMENT;
    if (sel_prev && sel_out &&
        spans_overlap(reinterpret_cast<const float*>(sel_prev), reinterpret_cast<const float*>(sel_out), p->groups_total))
        return HSADMM_ERR_INVALID_ARGUMENT;         // the repair pass reads the old record beside the new one
    if (out && (!out->packed || !out->layer_off || !out->kept_idx || !is_aligned(out->packed, 16) ||
                !is_aligned(out->layer_off, 8) || !is_aligned(out->kept_idx, 4)))
        return HSADMM_ERR_INVALID_ARGUMENT;
    if (!on_plan_device(p)) return HSADMM_ERR_INVALID_ARGUMENT;
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
    a.Ur = U; a.U = U_out ? U_out : U; a.Z = Z; a.Wbar = Wbar;
    a.key = sqnorm ? sqnorm : reinterpret_cast<double*>(ws + p->ws.key);
    a.colpart = reinterpret_cast<double*>(ws + p->ws.colpart);
    a.inv_R = 1.0f / (float)R;
    a.park_mean = R >= 3 ? 1 : 0;
    hipError_t e;
    // Under a prediction pass 1 writes the FILTER rows in the form their predicted fate makes final and packs the rows
    // it expects to be kept (and every row of the unconstrained layers).
    const bool hinted_chan = sel_prev != nullptr && U_out != nullptr && !p->items_chan.empty();   // CHANNEL layers too
    const bool hinted_both = sel_prev != nullptr && U_out != nullptr && !p->items_bfinal.empty(); // ... and BOTH layers
    const bool hinted = sel_prev != nullptr && (!p->items_plain.empty() || hinted_chan || hinted_both);
    const HintArgs h{sel_prev, out ? out->packed : nullptr, U_out ? 0 : 1, reinterpret_cast<int32_t*>(ws + p->ws.work),
                     p->d_layers};
    // Without a caller's prediction, a plan of FILTER and unconstrained layers whose dual is updated in place forms
    // one inside pass 1 (kernels_estimate.hpp).
    const bool est = !hinted && sel_prev == nullptr && U_out == nullptr && p->use_estimate;
    EstArgs ex{};
    if (est) {
        ex.pred = reinterpret_cast<int32_t*>(ws + p->ws.pred);
        ex.tag = reinterpret_cast<unsigned int*>(ws + p->ws.est_cnt);
        ex.keys = reinterpret_cast<double*>(ws + p->ws.est_keys);
        ex.thr = reinterpret_cast<double*>(ws + p->ws.est_thr);
        ex.thr_tag = reinterpret_cast<unsigned int*>(ws + p->ws.est_thr_tag);
        ex.layers = p->d_layers;
        ex.gen = const_cast<hsadmm_plan*>(p)->est_calls.fetch_add(1, std::memory_order_relaxed) + 1u;
        if (ex.gen == 0u)       // (the tag of a zeroed workspace: skipped when the counter wraps)
            ex.gen = const_cast<hsadmm_plan*>(p)->est_calls.fetch_add(1, std::memory_order_relaxed) + 1u;
    }
    WorkList wl{};
    if (hinted) {
        // the selection lists the row items the repair pass must visit, and hands out the offsets and kept lists itself
        wl.sel_prev = h.stash ? nullptr : sel_prev; wl.work = h.work; wl.pack = out ? 1 : 0;
        wl.channels = hinted_chan ? 1 : 0;
        wl.both = hinted_both ? 1 : 0;
        if (out) wl.co = CopyOut{out->layer_off, out->kept_idx};
        if (hinted_chan || hinted_both)      // (either implies the other where the plan has both kinds of layer)
            e = for_replica_count<true>(R, [&](auto c) {
                return launch(p, kPass1Hinted, project_pass1_hinted<decltype(c)::value, true>, (unsigned)p->items_proj.size(),
                              kBlock, s, (const WorkItem*)p->d_items_proj, a, (int)R, h);
            });
        else
            e = for_replica_count<true>(R, [&](auto c) {
                return launch(p, kPass1Hinted, project_pass1_hinted<decltype(c)::value>, (unsigned)p->items_proj.size(),
                              kBlock, s, (const WorkItem*)p->d_items_proj, a, (int)R, h);
            });
    } else if (est) {
        // the prediction is formed inside pass 1 and recorded for the repair pass; the selection hands out the offsets
        // and kept lists itself
        if (out) wl.co = CopyOut{out->layer_off, out->kept_idx};
        e = for_replica_count<true>(R, [&](auto c) {
            return launch(p, kPass1, project_pass1_est<decltype(c)::value>, (unsigned)p->items_est.size(), kBlock, s,
                          (const WorkItem*)p->d_items_est, a, (int)R, ex);
        });
    } else {
        e = for_replica_count<true>(R, [&](auto c) { return launch_pass1<decltype(c)::value>(p, a, R, s); });
    }
    if (e != hipSuccess) return HSADMM_ERR_HIP;
    // (the candidate of a BOTH layer is formed again from its parked mean and U)
    if (run_selection(p, a.key, a.colpart, a, mask, ws, s, sel_out, wl) != hipSuccess) return HSADMM_ERR_HIP;
    // The compaction of Z under the selection just made reads kept groups only, which FILTER layers hold in
    // final form since pass 1, so it shares a launch with the FILTER fix-up; the CHANNEL and BOTH layers are
    // packed by the pass that writes their Z.
    const bool fuse = out && !hinted && !est && !p->items_fix.empty();
    PackOut po{};
    po.pos = reinterpret_cast<const int32_t*>(ws + p->ws.pos);
    if (out) {
        po.cnt = reinterpret_cast<const int32_t*>(ws + p->ws.cnt);
        po.kept_idx = reinterpret_cast<const int32_t*>(ws + p->ws.kept_idx);
        po.layer_off = reinterpret_cast<const int64_t*>(ws + p->ws.layer_off);
        po.packed = out->packed;
        po.co = CopyOut{out->layer_off, out->kept_idx};
        po.n_layers = (int)p->layers.size();
    }
    if (hinted) {
        // every FILTER row from its predicted to its final form.  Dual in place: all row items (most hold a stash
        // to clear).  Dual out of place: as many workgroups as the device holds at once share the items the
        // selection listed.
        if (!p->items_fix.empty() || hinted_chan || hinted_both) {
            if (h.stash) {
                e = for_replica_count<true>(R, [&](auto c) {
                    return launch(p, kHintedRepair, hinted_repair_all<decltype(c)::value>, (unsigned)p->items_fix.size(),
                                  kBlock, s, (const WorkItem*)p->d_items_fix, a, (int)R, h, po);
                });
            } else {
                const unsigned n = (unsigned)std::min<size_t>(p->items_fix.size() + (hinted_chan ? p->items_chan.size() : 0) +
                                                                  (hinted_both ? p->items_bfinal.size() : 0), kRepairGrid);
                e = for_replica_count<true>(R, [&](auto c) {
                    return launch(p, kHintedRepair, hinted_repair<decltype(c)::value>, n, kBlock, s,
                                  (const WorkItem*)p->d_items_rows, a, (int)R, h, (const uint8_t*)mask, po);
                });
            }
            if (e != hipSuccess) return HSADMM_ERR_HIP;
        }
    } else if (est) {
        // every FILTER row from the form pass 1 chose to its final form (kept rows packed on the way) and, with a
        // compaction, the rows of the unconstrained layers gathered, in one launch
        const unsigned n_fix = (unsigned)p->items_fix.size();
        if (out)
            e = for_replica_count<true>(R, [&](auto c) {
                return launch(p, kFixupGather, fixup_gather_est<decltype(c)::value>, n_fix + (unsigned)p->items_none.size(),
                              kBlock, s, (const WorkItem*)p->d_items_fix, (int)n_fix, a, (int)R, (const int32_t*)ex.pred,
                              (const WorkItem*)p->d_items_none, po);
            });
        else
            e = for_replica_count<true>(R, [&](auto c) {
                return launch(p, kFixup, project_fixup_est<decltype(c)::value>, n_fix, kBlock, s,
                              (const WorkItem*)p->d_items_fix, a, (int)R, (const int32_t*)ex.pred, po.pos);
            });
        if (e != hipSuccess) return HSADMM_ERR_HIP;
    } else if (!p->items_fix.empty() && !fuse) {
        e = launch(p, kFixup, project_fixup, (unsigned)p->items_fix.size(), kBlock, s,
                   (const WorkItem*)p->d_items_fix, (const uint8_t*)mask, a.U, Z);
        if (e != hipSuccess) return HSADMM_ERR_HIP;
    }
    // Without FILTER layers the gather of the plain rows (unconstrained layers) has no fix-up to share a launch
    // with; it then rides on the last final pass.
    bool plain_pending = out && !fuse && !hinted && !est && !p->items_plain.empty();
    const unsigned n_plain = (unsigned)p->items_plain.size();
    if (!p->items_bfinal.empty() && !hinted_both) {
        // layers under both constraints: final Z and U from the parked mean and U, under both selections
        const unsigned gb = (unsigned)p->items_bfinal.size();
        if (out && plain_pending && p->items_chan.empty()) {
            e = launch(p, kBothFinal, final_gather<kMeanInZ>, gb + n_plain, kBlock, s,
                       (const WorkItem*)p->d_items_bfinal, (int)gb, a, 0, (const uint8_t*)mask, po,
                       (const WorkItem*)p->d_items_plain);
            plain_pending = false;
        } else if (out)
            e = launch(p, kBothFinal, project_frozen<kMeanInZ, true>, gb, kBlock, s, (const WorkItem*)p->d_items_bfinal,
                       a, 0, (const uint8_t*)mask, po);
        else
            e = launch(p, kBothFinal, project_frozen<kMeanInZ>, gb, kBlock, s, (const WorkItem*)p->d_items_bfinal,
                       a, 0, (const uint8_t*)mask, PackOut{});
        if (e != hipSuccess) return HSADMM_ERR_HIP;
    }
    if (!p->items_chan.empty() && !hinted_chan) {
        const uint8_t* cm = mask;
        const PackOut* pk = out ? &po : nullptr;
        const unsigned gc = (unsigned)p->items_chan.size();
        const WorkItem* ci = p->d_items_chan;
        const WorkItem* pi = p->d_items_plain;
        if (plain_pending) {
            switch (a.park_mean ? 0 : R) {
                case 0: e = launch(p, kChanFinal, final_gather<kMeanInZ>, gc + n_plain, kBlock, s, ci, (int)gc, a, (int)R, cm, po, pi); break;
                case 1: e = launch(p, kChanFinal, final_gather<1>, gc + n_plain, kBlock, s, ci, (int)gc, a, (int)R, cm, po, pi); break;
                default: e = launch(p, kChanFinal, final_gather<2>, gc + n_plain, kBlock, s, ci, (int)gc, a, (int)R, cm, po, pi); break;
            }
            plain_pending = false;
        } else {
            switch (a.park_mean ? 0 : R) {
                case 0: e = launch_channel_final<kMeanInZ>(p, a, R, cm, pk, s); break;
                case 1: e = launch_channel_final<1>(p, a, R, cm, pk, s); break;
                default: e = launch_channel_final<2>(p, a, R, cm, pk, s); break;
            }
        }
        if (e != hipSuccess) return HSADMM_ERR_HIP;
    }
    if (out && !p->items_plain.empty() && (fuse || plain_pending)) {
        const unsigned n_rows = (unsigned)p->items_plain.size();
        if (fuse)
            e = launch(p, kFixupGather, fixup_gather, (unsigned)p->items_fix.size() + n_rows, kBlock, s,
                       (const WorkItem*)p->d_items_fix, (int)p->items_fix.size(), (const uint8_t*)mask, a.U, Z,
                       (const WorkItem*)p->d_items_plain, po.pos, po.cnt, po.kept_idx, po.n_layers, po.layer_off,
                       po.packed, po.co);
        else
            e = launch(p, kGather, compact_gather<false>, n_rows, kBlock, s, (const WorkItem*)p->d_items_plain,
                       (const float*)Z, (const float*)nullptr, po.pos, po.cnt, po.kept_idx, po.n_layers,
                       po.layer_off, po.packed, po.co);
        if (e != hipSuccess) return HSADMM_ERR_HIP;
    }
    return HSADMM_OK;
}

int hsadmm_project(const hsadmm_plan_t* p, const float* const* W_replicas, int32_t R, float* U, float* Z,
                   float* Wbar, uint8_t* mask, double* sqnorm, void* workspace, size_t workspace_bytes,
                   void* hip_stream)
{
    return project_impl(p, W_replicas, R, U, Z, Wbar, mask, sqnorm, nullptr, workspace, workspace_bytes, hip_stream);
}

int hsadmm_project_compact(const hsadmm_plan_t* p, const float* const* W_replicas, int32_t R, float* U, float* Z,
                           float* Wbar, uint8_t* mask, double* sqnorm, float* packed, int64_t* layer_off,
                           int32_t* kept_idx, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    const CompactOut out{packed, layer_off, kept_idx};
    return project_impl(p, W_replicas, R, U, Z, Wbar, mask, sqnorm, &out, workspace, workspace_bytes, hip_stream);
}

int hsadmm_project_compact_static(const hsadmm_plan_t* p, const float* const* W_replicas, int32_t R, float* U,
                                  float* Z, float* Wbar, uint8_t* mask, double* sqnorm, float* packed,
                                  int64_t* layer_off, int32_t* kept_idx, void* hip_stream)
{
    if (!p) return HSADMM_ERR_INVALID_ARGUMENT;
    if (p->ws.total > kStaticScratchBytes) return HSADMM_ERR_UNSUPPORTED;     // the plan needs more scratch than the array holds
    const CompactOut out{packed, layer_off, kept_idx};
    // every kernel of the step writes the parts of the scratch it later reads, so nothing has to be cleared
    return project_impl(p, W_replicas, R, U, Z, Wbar, mask, sqnorm, &out, p->static_ws, kStaticScratchBytes, hip_stream);
}

int hsadmm_project_frozen(const hsadmm_plan_t* p, const float* const* W_replicas, int32_t R, float* U, float* Z,
                          float* Wbar, const uint8_t* mask, void* hip_stream)
{
    if (!p || !W_replicas || !U || !Z || !mask || R < 1) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!on_plan_device(p)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (R > HSADMM_MAX_REPLICAS) return HSADMM_ERR_UNSUPPORTED;
    if (!is_aligned(U, 16) || !is_aligned(Z, 16) || (Wbar && !is_aligned(Wbar, 16))) return HSADMM_ERR_INVALID_ARGUMENT;
    for (int r = 0; r < R; ++r)
        if (!W_replicas[r] || !is_aligned(W_replicas[r], 16)) return HSADMM_ERR_INVALID_ARGUMENT;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    ProjectArgs a{};
    for (int r = 0; r < R; ++r) a.W[r] = W_replicas[r];
    a.Ur = U; a.U = U; a.Z = Z; a.Wbar = Wbar;
    a.inv_R = 1.0f / (float)R;
    hipError_t e;
    e = for_replica_count<true>(R, [&](auto c) { return launch_frozen<decltype(c)::value>(p, a, R, mask, s); });
    return e == hipSuccess ? HSADMM_OK : HSADMM_ERR_HIP;
}

int hsadmm_project_frozen_compact(const hsadmm_plan_t* p, const float* const* W_replicas, int32_t R, float* U,
                                  float* Z, float* Wbar, const uint8_t* mask, int32_t mappings_cached, float* packed,
                                  int64_t* layer_off, int32_t* kept_idx, void* workspace, size_t workspace_bytes,
                                  void* hip_stream)
{
    if (!p || !W_replicas || !U || !Z || !mask || !packed || !layer_off || !kept_idx || !workspace || R < 1)
        return HSADMM_ERR_INVALID_ARGUMENT;
    if (!on_plan_device(p)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (R > HSADMM_MAX_REPLICAS) return HSADMM_ERR_UNSUPPORTED;
    if (!is_aligned(U, 16) || !is_aligned(Z, 16) || (Wbar && !is_aligned(Wbar, 16)) || !is_aligned(packed, 16) ||
        !is_aligned(layer_off, 8) || !is_aligned(kept_idx, 4) || !is_aligned(workspace, 256))
        return HSADMM_ERR_INVALID_ARGUMENT;
    for (int r = 0; r < R; ++r)
        if (!W_replicas[r] || !is_aligned(W_replicas[r], 16)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (workspace_bytes < p->ws.total) return HSADMM_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    if (!mappings_cached) {
        const int rc = run_scan(p, mask, ws, s);
        if (rc != HSADMM_OK) return rc;
    }
    ProjectArgs a{};
    for (int r = 0; r < R; ++r) a.W[r] = W_replicas[r];
    a.Ur = U; a.U = U; a.Z = Z; a.Wbar = Wbar;
    a.inv_R = 1.0f / (float)R;
    PackOut po{};
    po.pos = reinterpret_cast<const int32_t*>(ws + p->ws.pos);
    po.cnt = reinterpret_cast<const int32_t*>(ws + p->ws.cnt);
    po.kept_idx = reinterpret_cast<const int32_t*>(ws + p->ws.kept_idx);
    po.layer_off = reinterpret_cast<const int64_t*>(ws + p->ws.layer_off);
    po.packed = packed;
    po.co = CopyOut{layer_off, kept_idx};
    po.n_layers = (int)p->layers.size();
    hipError_t e;
    e = for_replica_count<true>(R, [&](auto c) { return launch_frozen_pack<decltype(c)::value>(p, a, R, mask, po, s); });
    if (e != hipSuccess) return HSADMM_ERR_HIP;
    return HSADMM_OK;
}

int hsadmm_mask_or(const hsadmm_plan_t* p, const uint8_t* const* masks, int32_t M, uint8_t* out, void* hip_stream)
{
    if (!p || !masks || !out || M < 1) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!on_plan_device(p)) return HSADMM_ERR_INVALID_ARGUMENT;
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

int hsadmm_mask_drift(const hsadmm_plan_t* p, const uint8_t* mask_a, const uint8_t* mask_b, int32_t* drift,
                      void* hip_stream)
{
    if (!p || !mask_a || !mask_b || !drift || !is_aligned(drift, 4)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!on_plan_device(p)) return HSADMM_ERR_INVALID_ARGUMENT;
    const hipError_t e = launch(p, kMaskDrift, mask_drift_kernel, (unsigned)p->layers.size(), kBlock,
                                static_cast<hipStream_t>(hip_stream), (const DevLayer*)p->d_layers, mask_a, mask_b,
                                drift);
    return e == hipSuccess ? HSADMM_OK : HSADMM_ERR_HIP;
}

static int compact_impl(const hsadmm_plan_t* p, const float* src, const float* src1, bool sum, const uint8_t* mask,
                        float* packed, int64_t* layer_off, int32_t* kept_idx, void* workspace,
                        size_t workspace_bytes, void* hip_stream)
{
    if (!p || !src || (sum && !src1) || !packed || !layer_off || !kept_idx || !workspace)
        return HSADMM_ERR_INVALID_ARGUMENT;
    if (!on_plan_device(p)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!is_aligned(src, 16) || (sum && !is_aligned(src1, 16)) || !is_aligned(packed, 16) ||
        !is_aligned(layer_off, 8) || !is_aligned(kept_idx, 4) || !is_aligned(workspace, 256))
        return HSADMM_ERR_INVALID_ARGUMENT;
    if (workspace_bytes < p->ws.total) return HSADMM_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    // The index mappings live in the workspace: derived from the mask here, or (mask == NULL) those the last
    // projection, compaction or expansion left there.  The gather hands the caller its copies.
    const int32_t* kidx = reinterpret_cast<const int32_t*>(ws + p->ws.kept_idx);
    CopyOut co{layer_off, kept_idx};
    if (mask) {
        const int rc = run_scan(p, mask, ws, s);
        if (rc != HSADMM_OK) return rc;
    }
    const int32_t* pos = reinterpret_cast<const int32_t*>(ws + p->ws.pos);
    const int32_t* cnt = reinterpret_cast<const int32_t*>(ws + p->ws.cnt);
    const int64_t* lo = reinterpret_cast<const int64_t*>(ws + p->ws.layer_off);
    hipError_t e;
    if (sum)
        e = launch(p, kGather, compact_gather<true>, (unsigned)p->items_rows.size(), kBlock, s,
                   (const WorkItem*)p->d_items_rows, src, src1, pos, cnt, kidx,
                   (int)p->layers.size(), lo, packed, co);
    else
        e = launch(p, kGather, compact_gather<false>, (unsigned)p->items_rows.size(), kBlock, s,
                   (const WorkItem*)p->d_items_rows, src, (const float*)nullptr, pos, cnt, kidx,
                   (int)p->layers.size(), lo, packed, co);
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
    if (rho1 == nullptr || rho2 == nullptr || a == nullptr || b == nullptr) return HSADMM_ERR_INVALID_ARGUMENT;
    if (L < 1 || M < 1 || P < 1) return HSADMM_ERR_INVALID_ARGUMENT;
    // Eq. (9): the three terms of gamma are the weight decay's share lambda / M, the P replicas' penalties and the
    // inter-node penalty.  Every layer is checked before the first weight is written.
    const double decay_share = lambda / static_cast<double>(M);
    const double replicas = static_cast<double>(P);
    auto gamma_of = [&](int32_t l) { return decay_share + replicas * rho1[l] + rho2[l]; };
    for (int32_t l = 0; l < L; ++l) {
        const bool penalties_ok = rho1[l] >= 0.0 && rho2[l] >= 0.0;
        if (!penalties_ok || !(gamma_of(l) > 0.0)) return HSADMM_ERR_INVALID_ARGUMENT;      // (a NaN fails one of them)
    }
    for (int32_t l = 0; l < L; ++l) {
        const double gamma = gamma_of(l);
        a[l] = static_cast<float>(replicas * rho1[l] / gamma);     // weight of Wbar + U
        b[l] = static_cast<float>(rho2[l] / gamma);                // weight of z - v
    }
    return HSADMM_OK;
}

int hsadmm_adapt_penalties(const double* residuals, int32_t L, int32_t P, int32_t n_out, double mu, double tau_incr,
                           double tau_decr, double rho1_max, double rho2_max, double* rho1, double* rho2,
                           float* scale_u, float* scale_v)
{
    if (!residuals || !rho1 || !rho2 || !scale_u || !scale_v || L < 1 || P < 1 || n_out < 1)
        return HSADMM_ERR_INVALID_ARGUMENT;
    if (!(mu > 0.0) || !(tau_incr >= 1.0) || !(tau_decr >= 1.0)) return HSADMM_ERR_INVALID_ARGUMENT;
    const double* sq_r[2] = {residuals, residuals + 2 * (size_t)L};                   // primal rows
    const double* sq_s[2] = {residuals + (size_t)L, residuals + 3 * (size_t)L};       // dual rows, without rho
    for (int32_t l = 0; l < L; ++l) {
        const bool rho_ok = rho1[l] > 0.0 && rho2[l] > 0.0 && rho1[l] <= rho1_max && rho2[l] <= rho2_max;
        const bool sums_ok = sq_r[0][l] >= 0.0 && sq_s[0][l] >= 0.0 && sq_r[1][l] >= 0.0 && sq_s[1][l] >= 0.0;
        if (!rho_ok || !sums_ok) return HSADMM_ERR_INVALID_ARGUMENT;                    // (NaN fails both)
    }
    // one penalty of one layer: the new value, and the factor its scaled dual takes
    auto balance = [&](double rho, double sum_r, double sum_s, double copies, double cap, float* scale) {
        const double norm_r = std::sqrt(sum_r);
        const double norm_s = rho * std::sqrt(copies * sum_s);
        double next = rho;
        if (norm_r > mu * norm_s) next = std::min(tau_incr * rho, cap);
        else if (norm_s > mu * norm_r) next = rho / tau_decr;
        *scale = (float)(rho / next);
        return next;
    };
    for (int32_t l = 0; l < L; ++l) {
        rho1[l] = balance(rho1[l], sq_r[0][l], sq_s[0][l], (double)P, rho1_max, &scale_u[l]);
        rho2[l] = balance(rho2[l], sq_r[1][l], sq_s[1][l], (double)n_out, rho2_max, &scale_v[l]);
    }
    return HSADMM_OK;
}

int hsadmm_scale_layers(const hsadmm_plan_t* p, float* X, const float* factor, void* hip_stream)
{
    if (!p || !X || !factor) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!on_plan_device(p)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!is_aligned(X, 16) || !is_aligned(factor, 4)) return HSADMM_ERR_INVALID_ARGUMENT;
    const hipError_t e = launch(p, kScaleLayers, scale_layers_kernel, (unsigned)p->items_rows.size(), kBlock,
                                static_cast<hipStream_t>(hip_stream), (const WorkItem*)p->d_items_rows, factor, X);
    return e == hipSuccess ? HSADMM_OK : HSADMM_ERR_HIP;
}

int hsadmm_plan_set_node_weights(hsadmm_plan_t* p, const float* a, const float* b)
{
    if (!p || !a || !b) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!on_plan_device(p)) return HSADMM_ERR_INVALID_ARGUMENT;
    const size_t L = p->layers.size();
    std::vector<float> ab;
    try {
        ab.resize(2 * L);
    } catch (...) {
        return HSADMM_ERR_HOST_MEMORY;
    }
    for (size_t l = 0; l < L; ++l) { ab[2 * l] = a[l]; ab[2 * l + 1] = b[l]; }
    if (hipMemcpy(p->d_coef, ab.data(), sizeof(float) * ab.size(), hipMemcpyHostToDevice) != hipSuccess)
        return HSADMM_ERR_HIP;
    return HSADMM_OK;
}

// coef_arg: device, 2L floats a_0, b_0, a_1, b_1, ... (null: the weights stored in the plan)
static int project_weighted_impl(const hsadmm_plan_t* p, const float* const* W_replicas, int32_t R, float* U,
                                 const float* Zg, const float* Vd, float* Z, float* Wbar, uint8_t* mask,
                                 double* sqnorm, const CompactOut* out, void* workspace, size_t workspace_bytes,
                                 void* hip_stream, const float* coef_arg = nullptr, int32_t* sel_out = nullptr,
                                 const float* Zi_prev = nullptr, double* residuals = nullptr,
                                 const int32_t* sel_prev = nullptr, float* U_out = nullptr)
{
    if (!p || !W_replicas || !U || !Zg || !Vd || !Z || !mask || !workspace || R < 1) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!is_aligned(coef_arg, 4) || !is_aligned(sel_out, 4) || !is_aligned(sel_prev, 4) || !is_aligned(U_out, 16))
        return HSADMM_ERR_INVALID_ARGUMENT;
    if (U_out && (spans_overlap(U_out, U, p->arena_elems) || spans_overlap(U_out, Z, p->arena_elems) ||
                  spans_overlap(U_out, Zg, p->arena_elems) || spans_overlap(U_out, Vd, p->arena_elems)))
        return HSADMM_ERR_INVALID_ARGUMENT;
    if (sel_prev && sel_out &&
        spans_overlap(reinterpret_cast<const float*>(sel_prev), reinterpret_cast<const float*>(sel_out), p->groups_total))
        return HSADMM_ERR_INVALID_ARGUMENT;
    // a prediction needs the old dual to stay readable (a wrong one is repaired from the inputs)
    if (sel_prev && !U_out) return HSADMM_ERR_UNSUPPORTED;
    // the intra-node residual norms on the way: both or neither of the previous z_i and the place for the norms
    if ((Zi_prev == nullptr) != (residuals == nullptr)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (residuals && (!is_aligned(Zi_prev, 16) || !is_aligned(residuals, 8) || spans_overlap(Zi_prev, Z, p->arena_elems) ||
                      spans_overlap(Zi_prev, U, p->arena_elems) || (U_out && spans_overlap(Zi_prev, U_out, p->arena_elems))))
        return HSADMM_ERR_INVALID_ARGUMENT;
    const float* const coef = coef_arg ? coef_arg : p->d_coef;
    if (out && (!out->packed || !out->layer_off || !out->kept_idx || !is_aligned(out->packed, 16) ||
                !is_aligned(out->layer_off, 8) || !is_aligned(out->kept_idx, 4)))
        return HSADMM_ERR_INVALID_ARGUMENT;
    if (!on_plan_device(p)) return HSADMM_ERR_INVALID_ARGUMENT;
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
    w.p.Ur = U; w.p.U = U_out ? U_out : U; w.p.Z = Z; w.p.Wbar = Wbar;
    w.p.key = sqnorm ? sqnorm : reinterpret_cast<double*>(ws + p->ws.key);
    w.p.colpart = reinterpret_cast<double*>(ws + p->ws.colpart);
    w.p.inv_R = 1.0f / (float)R;
    w.p.park_mean = R >= 3 ? 1 : 0;
    w.p.Zg = Zg; w.p.Vd = Vd; w.p.coef = coef;
    w.Zg = Zg; w.Vd = Vd; w.coef = coef;
    w.Zi_prev = Zi_prev;
    w.rowres = reinterpret_cast<double*>(ws + p->ws.rowres);
    const unsigned grid = (unsigned)p->items_proj.size();
    const WorkItem* items = p->d_items_proj;
    hipError_t e;
    // (a prediction comes with the dual out of place here, so every mode can take it)
    const bool hinted_tiles = sel_prev != nullptr && (!p->items_chan.empty() || !p->items_bfinal.empty());
    const bool hinted = sel_prev != nullptr && (!p->items_plain.empty() || hinted_tiles);
    const WeightedHint wh{sel_prev, out ? out->packed : nullptr, reinterpret_cast<int32_t*>(ws + p->ws.work), p->d_layers};
    WorkList wl{};
    if (hinted) {
        wl.sel_prev = sel_prev; wl.work = wh.work; wl.pack = out ? 1 : 0;
        wl.channels = wl.both = hinted_tiles ? 1 : 0;
        if (out) wl.co = CopyOut{out->layer_off, out->kept_idx};
        const int form = (residuals ? 1 : 0) | (hinted_tiles ? 2 : 0);
        e = for_replica_count<false>(R, [&](auto c) {
            constexpr int RC = decltype(c)::value;
            switch (form) {
                case 0: return launch(p, kWKeys, weighted_pass1_hinted<RC, false, false>, grid, kBlock, s, items, w, (int)R, wh);
                case 1: return launch(p, kWKeys, weighted_pass1_hinted<RC, true, false>, grid, kBlock, s, items, w, (int)R, wh);
                case 2: return launch(p, kWKeys, weighted_pass1_hinted<RC, false, true>, grid, kBlock, s, items, w, (int)R, wh);
                default: return launch(p, kWKeys, weighted_pass1_hinted<RC, true, true>, grid, kBlock, s, items, w, (int)R, wh);
            }
        });
    } else if (residuals)
        e = for_replica_count<false>(R, [&](auto c) {
            return launch(p, kWKeys, weighted_pass1<decltype(c)::value, true>, grid, kBlock, s, items, w, (int)R);
        });
    else
        e = for_replica_count<false>(R, [&](auto c) {
            return launch(p, kWKeys, weighted_pass1<decltype(c)::value>, grid, kBlock, s, items, w, (int)R);
        });
    if (e != hipSuccess) return HSADMM_ERR_HIP;
    // (the weighted candidate of a BOTH layer is formed again from its parked mean, U, Zg and Vd)
    if (residuals) { wl.rowres = w.rowres; wl.res_out = residuals; }       // FILTER / unconstrained layers: rows 0 and 1
    if (run_selection(p, w.p.key, w.p.colpart, w.p, mask, ws, s, sel_out, wl) != hipSuccess) return HSADMM_ERR_HIP;
    const uint8_t* cm = mask;
    PackOut po{};
    if (out) {
        po.pos = reinterpret_cast<const int32_t*>(ws + p->ws.pos);
        po.cnt = reinterpret_cast<const int32_t*>(ws + p->ws.cnt);
        po.kept_idx = reinterpret_cast<const int32_t*>(ws + p->ws.kept_idx);
        po.layer_off = reinterpret_cast<const int64_t*>(ws + p->ws.layer_off);
        po.packed = out->packed;
        po.co = CopyOut{out->layer_off, out->kept_idx};
        po.n_layers = (int)p->layers.size();
    }
    // With a compaction to follow, the FILTER fix-up packs its kept rows as it forms them and shares its launch with
    // the gather of the unconstrained layers' rows; CHANNEL and BOTH layers are packed by their final pass.
    const bool fuse = out && !hinted && !p->items_fix.empty();
    if (hinted) {
        // FILTER rows are final unless their prediction was wrong (or, packed, their rank moved), CHANNEL and BOTH
        // layers unless their selection differs from the record: the listed items
        if (!p->items_fix.empty() || hinted_tiles) {
            const unsigned n = (unsigned)std::min<size_t>(p->items_fix.size() + p->items_chan.size() + p->items_bfinal.size(),
                                                          kRepairGrid);
            const int32_t* pos = reinterpret_cast<const int32_t*>(ws + p->ws.pos);
            e = for_replica_count<false>(R, [&](auto c) {
                return launch(p, kWHintedRepair, weighted_hinted_repair<decltype(c)::value>, n, kBlock, s,
                              (const WorkItem*)p->d_items_rows, w, (int)R, wh, pos, cm, po);
            });
            if (e != hipSuccess) return HSADMM_ERR_HIP;
        }
    } else if (!p->items_fix.empty() && !fuse) {
        e = launch(p, kWFixup, weighted_fixup, (unsigned)p->items_fix.size(), kBlock, s,
                   (const WorkItem*)p->d_items_fix, cm, w.p.U, Z, Zg, Vd, coef);
        if (e != hipSuccess) return HSADMM_ERR_HIP;
    }
    // Final pass of the CHANNEL and BOTH layers: the frozen-mask kernel in its weighted form, on the parked mean
    // where pass 1 parked it (BOTH always, CHANNEL with 3 or more replicas), else on the replicas.
    if (!p->items_bfinal.empty() && !hinted_tiles) {
        const unsigned gb = (unsigned)p->items_bfinal.size();
        const WorkItem* bi = p->d_items_bfinal;
        if (out) e = launch(p, kWFinal, project_frozen<kMeanInZ, true, true>, gb, kBlock, s, bi, w.p, 0, cm, po);
        else e = launch(p, kWFinal, project_frozen<kMeanInZ, false, true>, gb, kBlock, s, bi, w.p, 0, cm, PackOut{});
        if (e != hipSuccess) return HSADMM_ERR_HIP;
    }
    if (!p->items_chan.empty() && !hinted_tiles) {
        const unsigned gc = (unsigned)p->items_chan.size();
        const WorkItem* ci = p->d_items_chan;
        const int sel = w.p.park_mean ? 0 : (int)R;          // 0: parked mean; else R is 1 or 2
        if (out) {
            if (sel == 0) e = launch(p, kWFinal, project_frozen<kMeanInZ, true, true>, gc, kBlock, s, ci, w.p, (int)R, cm, po);
            else if (sel == 1) e = launch(p, kWFinal, project_frozen<1, true, true>, gc, kBlock, s, ci, w.p, (int)R, cm, po);
            else e = launch(p, kWFinal, project_frozen<2, true, true>, gc, kBlock, s, ci, w.p, (int)R, cm, po);
        } else {
            if (sel == 0) e = launch(p, kWFinal, project_frozen<kMeanInZ, false, true>, gc, kBlock, s, ci, w.p, (int)R, cm, PackOut{});
            else if (sel == 1) e = launch(p, kWFinal, project_frozen<1, false, true>, gc, kBlock, s, ci, w.p, (int)R, cm, PackOut{});
            else e = launch(p, kWFinal, project_frozen<2, false, true>, gc, kBlock, s, ci, w.p, (int)R, cm, PackOut{});
        }
        if (e != hipSuccess) return HSADMM_ERR_HIP;
    }
    if (out && !hinted) {
        if (fuse)
            e = launch(p, kWFixupPack, weighted_fixup_pack, (unsigned)(p->items_fix.size() + p->items_none.size()),
                       kBlock, s, (const WorkItem*)p->d_items_fix, (int)p->items_fix.size(), cm, w.p.U, Z, Zg, Vd,
                       coef, (const WorkItem*)p->d_items_none, po);
        else if (!p->items_none.empty())
            e = launch(p, kGather, compact_gather<true>, (unsigned)p->items_none.size(), kBlock, s,
                       (const WorkItem*)p->d_items_none, (const float*)Z, Vd, po.pos, po.cnt, po.kept_idx,
                       po.n_layers, po.layer_off, po.packed, po.co);
        if (e != hipSuccess) return HSADMM_ERR_HIP;
    }
    if (residuals) {
        // (the selection has added up rows 0 and 1 of the FILTER and unconstrained layers)
        // CHANNEL and BOTH layers: their share of rows 0 and 1 from a pass over their final values
        double* part = reinterpret_cast<double*>(ws + p->ws.respart);
        if (!p->items_chan.empty() || !p->items_bfinal.empty()) {
            ResidualArgs ra{};
            for (int r = 0; r < R; ++r) ra.W[r] = W_replicas[r];
            ra.Zi = Z; ra.Zi_prev = Zi_prev; ra.part = part;
            e = for_replica_count<false>(R, [&](auto c) {
                return launch(p, kResPart, residual_partials<decltype(c)::value>, (unsigned)p->items_rows.size(), kBlock,
                              s, (const WorkItem*)p->d_items_rows, ra, (int)R,
                              (1 << HSADMM_MODE_CHANNEL) | (1 << HSADMM_MODE_BOTH));
            });
            if (e != hipSuccess) return HSADMM_ERR_HIP;
            e = launch(p, kResPick, residual_pick, (unsigned)p->layers.size(), kBlock, s, (const DevLayer*)p->d_layers,
                       (int)p->layers.size(), (const double*)part, residuals);
            if (e != hipSuccess) return HSADMM_ERR_HIP;
        }
    }
    return HSADMM_OK;
}

int hsadmm_project_weighted(const hsadmm_plan_t* p, const float* const* W_replicas, int32_t R, float* U,
                            const float* Zg, const float* Vd, float* Z, float* Wbar, uint8_t* mask, double* sqnorm,
                            void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return project_weighted_impl(p, W_replicas, R, U, Zg, Vd, Z, Wbar, mask, sqnorm, nullptr, workspace,
                                 workspace_bytes, hip_stream);
}

int hsadmm_project_weighted_compact(const hsadmm_plan_t* p, const float* const* W_replicas, int32_t R, float* U,
                                    const float* Zg, const float* Vd, float* Z, float* Wbar, uint8_t* mask,
                                    double* sqnorm, float* packed, int64_t* layer_off, int32_t* kept_idx,
                                    void* workspace, size_t workspace_bytes, void* hip_stream)
{
    const CompactOut out{packed, layer_off, kept_idx};
    return project_weighted_impl(p, W_replicas, R, U, Zg, Vd, Z, Wbar, mask, sqnorm, &out, workspace,
                                 workspace_bytes, hip_stream);
}

// The retraining branch with the full candidate: one pass of the frozen-mask kernel in its weighted form over every
// layer's row items; with `out` it also packs c = z_i + v_i under the mask's index mappings.
static int weighted_frozen_impl(const hsadmm_plan_t* p, const float* const* W_replicas, int32_t R, float* U,
                                const float* Zg, const float* Vd, float* Z, float* Wbar, const uint8_t* mask,
                                const CompactOut* out, int32_t mappings_cached, void* workspace,
                                size_t workspace_bytes, void* hip_stream, double* residuals = nullptr,
                                bool with_residuals = false, const float* coef_arg = nullptr)
{
    if (!p || !W_replicas || !U || !Zg || !Vd || !Z || !mask || R < 1) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!is_aligned(coef_arg, 4)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (with_residuals && (!out || !residuals || !is_aligned(residuals, 8))) return HSADMM_ERR_INVALID_ARGUMENT;
    if (out && (!out->packed || !out->layer_off || !out->kept_idx || !workspace || !is_aligned(out->packed, 16) ||
                !is_aligned(out->layer_off, 8) || !is_aligned(out->kept_idx, 4) || !is_aligned(workspace, 256)))
        return HSADMM_ERR_INVALID_ARGUMENT;
    if (!on_plan_device(p)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (R > HSADMM_MAX_REPLICAS) return HSADMM_ERR_UNSUPPORTED;
    if (!is_aligned(U, 16) || !is_aligned(Z, 16) || !is_aligned(Zg, 16) || !is_aligned(Vd, 16) ||
        (Wbar && !is_aligned(Wbar, 16)))
        return HSADMM_ERR_INVALID_ARGUMENT;
    for (int r = 0; r < R; ++r)
        if (!W_replicas[r] || !is_aligned(W_replicas[r], 16)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (out && workspace_bytes < p->ws.total) return HSADMM_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    ProjectArgs a{};
    for (int r = 0; r < R; ++r) a.W[r] = W_replicas[r];
    a.Ur = U; a.U = U; a.Z = Z; a.Wbar = Wbar;
    a.inv_R = 1.0f / (float)R;
    a.Zg = Zg; a.Vd = Vd; a.coef = coef_arg ? coef_arg : p->d_coef;
    PackOut po{};
    if (out) {
        if (!mappings_cached) {
            const int rc = run_scan(p, mask, ws, s);
            if (rc != HSADMM_OK) return rc;
        }
        po.pos = reinterpret_cast<const int32_t*>(ws + p->ws.pos);
        po.cnt = reinterpret_cast<const int32_t*>(ws + p->ws.cnt);
        po.kept_idx = reinterpret_cast<const int32_t*>(ws + p->ws.kept_idx);
        po.layer_off = reinterpret_cast<const int64_t*>(ws + p->ws.layer_off);
        po.packed = out->packed;
        po.co = CopyOut{out->layer_off, out->kept_idx};
        po.n_layers = (int)p->layers.size();
    }
    const unsigned grid = (unsigned)p->items_rows.size();
    const WorkItem* items = p->d_items_rows;
    hipError_t e;
    if (with_residuals) {
        a.respart = reinterpret_cast<double*>(ws + p->ws.respart);
        e = for_replica_count<false>(R, [&](auto c) {
            return launch(p, kRetrainProject, project_frozen<decltype(c)::value, true, true, true>, grid, kBlock, s, items, a,
                          (int)R, mask, po);
        });
        if (e != hipSuccess) return HSADMM_ERR_HIP;
        e = launch(p, kResFinish, residual_finish, (unsigned)p->layers.size(), kBlock, s, (const DevLayer*)p->d_layers,
                   (int)p->layers.size(), (const double*)a.respart, residuals, 0, 2);
    } else if (out) {
        e = for_replica_count<false>(R, [&](auto c) {
            return launch(p, kFrozen, project_frozen<decltype(c)::value, true, true>, grid, kBlock, s, items, a, (int)R, mask,
                          po);
        });
    } else {
        e = for_replica_count<false>(R, [&](auto c) {
            return launch(p, kFrozen, project_frozen<decltype(c)::value, false, true>, grid, kBlock, s, items, a, (int)R, mask,
                          po);
        });
    }
    return e == hipSuccess ? HSADMM_OK : HSADMM_ERR_HIP;
}

int hsadmm_project_weighted_frozen(const hsadmm_plan_t* p, const float* const* W_replicas, int32_t R, float* U,
                                   const float* Zg, const float* Vd, float* Z, float* Wbar, const uint8_t* mask,
                                   void* hip_stream)
{
    return weighted_frozen_impl(p, W_replicas, R, U, Zg, Vd, Z, Wbar, mask, nullptr, 0, nullptr, 0, hip_stream);
}

int hsadmm_project_weighted_frozen_compact(const hsadmm_plan_t* p, const float* const* W_replicas, int32_t R,
                                           float* U, const float* Zg, const float* Vd, float* Z, float* Wbar,
                                           const uint8_t* mask, int32_t mappings_cached, float* packed,
                                           int64_t* layer_off, int32_t* kept_idx, void* workspace,
                                           size_t workspace_bytes, void* hip_stream)
{
    const CompactOut out{packed, layer_off, kept_idx};
    return weighted_frozen_impl(p, W_replicas, R, U, Zg, Vd, Z, Wbar, mask, &out, mappings_cached, workspace,
                                workspace_bytes, hip_stream);
}

int hsadmm_retrain_project(const hsadmm_plan_t* p, const float* const* W_replicas, int32_t R, float* U,
                           const float* Zg, const float* Vd, float* Z, float* Wbar, const uint8_t* mask,
                           int32_t mappings_cached, float* packed, int64_t* layer_off, int32_t* kept_idx,
                           double* residuals, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    const CompactOut out{packed, layer_off, kept_idx};
    return weighted_frozen_impl(p, W_replicas, R, U, Zg, Vd, Z, Wbar, mask, &out, mappings_cached, workspace,
                                workspace_bytes, hip_stream, residuals, true);
}

int hsadmm_step(const hsadmm_plan_t* p, const hsadmm_step_args_t* x)
{
    if (!p || !x || x->struct_bytes != sizeof(hsadmm_step_args_t)) return HSADMM_ERR_INVALID_ARGUMENT;
    const bool weighted = x->Zg != nullptr || x->Vd != nullptr;          // both are required then (checked below)
    const bool frozen = x->mask_frozen != nullptr;
    const bool pack = x->packed != nullptr || x->layer_off != nullptr || x->kept_idx != nullptr;
    if (!weighted && x->coef) return HSADMM_ERR_INVALID_ARGUMENT;        // weights without the terms they weigh
    const CompactOut out{x->packed, x->layer_off, x->kept_idx};         // (each impl wants all three or none)
    if (x->U_out && frozen) return HSADMM_ERR_UNSUPPORTED;               // that pass updates the dual in place
    if (frozen) {
        // retraining branch: the given mask replaces the selection; nothing is selected, predicted or recorded
        if (x->mask || x->sqnorm || x->sel_prev || x->sel) return HSADMM_ERR_INVALID_ARGUMENT;
        if (x->residuals && !(weighted && pack)) return HSADMM_ERR_UNSUPPORTED;
        if (x->Zi_prev) return HSADMM_ERR_INVALID_ARGUMENT;              // (under a frozen support Z itself brings the previous z_i)
        if (weighted)
            return weighted_frozen_impl(p, x->W_replicas, x->R, x->U, x->Zg, x->Vd, x->Z, x->Wbar, x->mask_frozen,
                                        pack ? &out : nullptr, x->mappings_cached, x->workspace, x->workspace_bytes,
                                        x->hip_stream, x->residuals, x->residuals != nullptr, x->coef);
        if (pack)
            return hsadmm_project_frozen_compact(p, x->W_replicas, x->R, x->U, x->Z, x->Wbar, x->mask_frozen,
                                                 x->mappings_cached, x->packed, x->layer_off, x->kept_idx,
                                                 x->workspace, x->workspace_bytes, x->hip_stream);
        return hsadmm_project_frozen(p, x->W_replicas, x->R, x->U, x->Z, x->Wbar, x->mask_frozen, x->hip_stream);
    }
    if (x->mappings_cached) return HSADMM_ERR_UNSUPPORTED;
    if (x->residuals && !weighted) return HSADMM_ERR_UNSUPPORTED;          // (for the plain candidate: hsadmm_residuals)
    if (weighted)
        return project_weighted_impl(p, x->W_replicas, x->R, x->U, x->Zg, x->Vd, x->Z, x->Wbar, x->mask, x->sqnorm,
                                     pack ? &out : nullptr, x->workspace, x->workspace_bytes, x->hip_stream, x->coef,
                                     x->sel, x->Zi_prev, x->residuals, x->sel_prev, x->U_out);
    return project_impl(p, x->W_replicas, x->R, x->U, x->Z, x->Wbar, x->mask, x->sqnorm, pack ? &out : nullptr,
                        x->workspace, x->workspace_bytes, x->hip_stream, x->sel_prev, x->sel, x->U_out);
}

int hsadmm_selection_from_mask(const hsadmm_plan_t* p, const uint8_t* mask, int32_t* sel, void* workspace,
                               size_t workspace_bytes, void* hip_stream)
{
    if (!p || !mask || !sel || !workspace || !is_aligned(sel, 4) || !is_aligned(workspace, 256))
        return HSADMM_ERR_INVALID_ARGUMENT;
    if (!on_plan_device(p)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (workspace_bytes < p->ws.total) return HSADMM_ERR_WORKSPACE;
    return run_scan(p, mask, static_cast<char*>(workspace), static_cast<hipStream_t>(hip_stream), sel);
}

int hsadmm_residuals(const hsadmm_plan_t* p, const float* const* W_replicas, int32_t R, const float* Zi,
                     const float* Zi_prev, const float* Zg, const float* Zg_prev, double* out, void* workspace,
                     size_t workspace_bytes, void* hip_stream)
{
    if (!p || !W_replicas || !Zi || !out || !workspace || R < 1) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!on_plan_device(p)) return HSADMM_ERR_INVALID_ARGUMENT;
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
    e = for_replica_count<false>(R, [&](auto c) {
        return launch(p, kResPart, residual_partials<decltype(c)::value>, grid, kBlock, s, items, a, (int)R, 0xf);
    });
    if (e != hipSuccess) return HSADMM_ERR_HIP;
    e = launch(p, kResFinish, residual_finish, (unsigned)p->layers.size(), kBlock, s,
               (const DevLayer*)p->d_layers, (int)p->layers.size(), (const double*)a.part, out, 0, 4);
    return e == hipSuccess ? HSADMM_OK : HSADMM_ERR_HIP;
}

int hsadmm_layer_sqnorms(const hsadmm_plan_t* p, const float* X, double* out, void* workspace, size_t workspace_bytes,
                         void* hip_stream)
{
    if (!p || !X || !out || !workspace) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!on_plan_device(p)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!is_aligned(X, 16) || !is_aligned(out, 8) || !is_aligned(workspace, 256)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (workspace_bytes < p->ws.total) return HSADMM_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    double* part = reinterpret_cast<double*>(static_cast<char*>(workspace) + p->ws.respart);
    hipError_t e = launch(p, kSqnormPart, sqnorm_partials, (unsigned)p->items_rows.size(), kBlock, s,
                          (const WorkItem*)p->d_items_rows, X, part);
    if (e != hipSuccess) return HSADMM_ERR_HIP;
    e = launch(p, kResFinish, residual_finish, (unsigned)p->layers.size(), kBlock, s, (const DevLayer*)p->d_layers,
               (int)p->layers.size(), (const double*)part, out, 0, 1);
    return e == hipSuccess ? HSADMM_OK : HSADMM_ERR_HIP;
}

int hsadmm_stopping_test(const int64_t* n_elems, int32_t n_layers, int32_t P, int32_t n_out, const double* rho1,
                         const double* rho2, const double* residuals, const double* magnitudes, double eps_abs,
                         double eps_rel, int32_t* layer_done, int32_t* all_done)
{
    if (!n_elems || !rho1 || !rho2 || !residuals || !magnitudes || !layer_done || !all_done || n_layers < 1 || P < 1 ||
        n_out < 1)
        return HSADMM_ERR_INVALID_ARGUMENT;
    if (!(eps_abs >= 0.0) || !(eps_rel >= 0.0)) return HSADMM_ERR_INVALID_ARGUMENT;
    const size_t L = (size_t)n_layers;
    auto row = [L](const double* table, int r, size_t l) { return table[(size_t)r * L + l]; };
    for (size_t l = 0; l < L; ++l) {                       // everything is checked before the first flag is written
        bool ok = n_elems[l] >= 1 && rho1[l] > 0.0 && rho2[l] > 0.0;
        for (int r = 0; r < 4 && ok; ++r) ok = row(residuals, r, l) >= 0.0;
        for (int r = 0; r < 5 && ok; ++r) ok = row(magnitudes, r, l) >= 0.0;
        if (!ok) return HSADMM_ERR_INVALID_ARGUMENT;       // (a NaN fails its comparison)
    }
    const double replicas = (double)P, nodes = (double)n_out;
    int32_t open_layers = 0;
    for (size_t l = 0; l < L; ++l) {
        const double elems = (double)n_elems[l];
        const double w1 = rho1[l] * rho1[l], w2 = rho2[l] * rho2[l];
        // squared norms of the stacked residuals of both consensus levels, and of the stacks the tolerances scale with
        const double primal_sq = row(residuals, 0, l) + row(residuals, 2, l);
        const double dual_sq = replicas * w1 * row(residuals, 1, l) + nodes * w2 * row(residuals, 3, l);
        const double first_vars_sq = row(magnitudes, 0, l) + row(magnitudes, 1, l);                   // theta_j's and z_i
        const double second_vars_sq = replicas * row(magnitudes, 1, l) + nodes * row(magnitudes, 2, l);  // z_i per replica, z
        const double duals_sq = w1 * row(magnitudes, 3, l) + w2 * row(magnitudes, 4, l);              // rho_1 u_j, rho_2 v_i
        const double absolute = std::sqrt((replicas + 1.0) * elems * nodes) * eps_abs;
        const double tol_primal = absolute + eps_rel * std::sqrt(std::max(first_vars_sq, second_vars_sq));
        const double tol_dual = absolute + eps_rel * std::sqrt(duals_sq);
        const bool done = std::sqrt(primal_sq) < tol_primal && std::sqrt(dual_sq) < tol_dual;
        layer_done[l] = done ? 1 : 0;
        open_layers += done ? 0 : 1;
    }
    *all_done = open_layers == 0 ? 1 : 0;
    return HSADMM_OK;
}

int hsadmm_dual_inter(const hsadmm_plan_t* p, const float* Zi, const float* Zg, float* Vd, void* hip_stream)
{
    if (!p || !Zi || !Zg || !Vd) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!on_plan_device(p)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!is_aligned(Zi, 16) || !is_aligned(Zg, 16) || !is_aligned(Vd, 16)) return HSADMM_ERR_INVALID_ARGUMENT;
    const hipError_t e = launch(p, kDualInter, dual_inter_kernel, (unsigned)p->items_rows.size(), kBlock,
                                static_cast<hipStream_t>(hip_stream), (const WorkItem*)p->d_items_rows, Zi, Zg, Vd);
    return e == hipSuccess ? HSADMM_OK : HSADMM_ERR_HIP;
}

int hsadmm_average(const hsadmm_plan_t* p, const float* const* bufs, int32_t M, int64_t n_elems, float* out,
                   void* hip_stream)
{
    if (!p || !bufs || !out || M < 1 || n_elems < 0) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!on_plan_device(p)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (M > HSADMM_MAX_MASKS) return HSADMM_ERR_UNSUPPORTED;
    if (!is_aligned(out, 16)) return HSADMM_ERR_INVALID_ARGUMENT;
    AverageArgs a{};
    for (int i = 0; i < M; ++i) {
        if (!bufs[i] || !is_aligned(bufs[i], 16)) return HSADMM_ERR_INVALID_ARGUMENT;
        a.b[i] = bufs[i];
    }
    if (n_elems == 0) return HSADMM_OK;
    int64_t want = ((n_elems >> 2) + kBlock - 1) / kBlock;      // one quad per thread ...
    if (want > 16384) want = 16384;                              // ... up to a grid that fills the device many times
    if (want < 1) want = 1;
    const hipError_t e = launch(p, kAverage, average_kernel, (unsigned)want, kBlock, static_cast<hipStream_t>(hip_stream),
                                a, (int)M, 1.0f / (float)M, n_elems, out);
    return e == hipSuccess ? HSADMM_OK : HSADMM_ERR_HIP;
}

static int expand_impl(const hsadmm_plan_t* p, const float* packed, const uint8_t* mask, float* dst, const float* Zi,
                       float* Vd, bool dual, void* workspace, size_t workspace_bytes, void* hip_stream,
                       const float* z_prev = nullptr, double* residuals = nullptr, bool with_residuals = false)
{
    if (!p || !packed || !dst || !workspace || (dual && (!Zi || !Vd))) return HSADMM_ERR_INVALID_ARGUMENT;
    if (with_residuals && (!dual || !z_prev || !residuals || !is_aligned(z_prev, 16) || !is_aligned(residuals, 8) ||
                           spans_overlap(z_prev, dst, p->arena_elems) || spans_overlap(z_prev, Vd, p->arena_elems)))
        return HSADMM_ERR_INVALID_ARGUMENT;
    if (!on_plan_device(p)) return HSADMM_ERR_INVALID_ARGUMENT;
    if (!is_aligned(packed, 16) || !is_aligned(dst, 16) || !is_aligned(workspace, 256) ||
        (dual && (!is_aligned(Zi, 16) || !is_aligned(Vd, 16))))
        return HSADMM_ERR_INVALID_ARGUMENT;
    if (workspace_bytes < p->ws.total) return HSADMM_ERR_WORKSPACE;
    hipStream_t s = static_cast<hipStream_t>(hip_stream);
    char* ws = static_cast<char*>(workspace);
    const int64_t* lo = reinterpret_cast<const int64_t*>(ws + p->ws.layer_off);
    if (mask) {
        const int rc = run_scan(p, mask, ws, s);
        if (rc != HSADMM_OK) return rc;
    }   // else: the index mappings already held in this workspace are used
    const int32_t* pos = reinterpret_cast<const int32_t*>(ws + p->ws.pos);
    const int32_t* cnt = reinterpret_cast<const int32_t*>(ws + p->ws.cnt);
    if (with_residuals) {
        double* part = reinterpret_cast<double*>(ws + p->ws.respart);
        hipError_t e = launch(p, kRetrainExpand, expand_scatter<true, true>, (unsigned)p->items_rows.size(), kBlock, s,
                              (const WorkItem*)p->d_items_rows, packed, pos, cnt, (int)p->layers.size(), lo, dst, Zi, Vd,
                              z_prev, part);
        if (e != hipSuccess) return HSADMM_ERR_HIP;
        e = launch(p, kResFinish, residual_finish, (unsigned)p->layers.size(), kBlock, s, (const DevLayer*)p->d_layers,
                   (int)p->layers.size(), (const double*)part, residuals, 2, 4);
        return e == hipSuccess ? HSADMM_OK : HSADMM_ERR_HIP;
    }
    const hipError_t e = dual
        ? launch(p, kScatter, expand_scatter<true>, (unsigned)p->items_rows.size(), kBlock, s,
                 (const WorkItem*)p->d_items_rows, packed, pos, cnt, (int)p->layers.size(), lo, dst, Zi, Vd,
                 (const float*)nullptr, (double*)nullptr)
        : launch(p, kScatter, expand_scatter<false>, (unsigned)p->items_rows.size(), kBlock, s,
                 (const WorkItem*)p->d_items_rows, packed, pos, cnt, (int)p->layers.size(), lo, dst,
                 (const float*)nullptr, (float*)nullptr, (const float*)nullptr, (double*)nullptr);
    return e == hipSuccess ? HSADMM_OK : HSADMM_ERR_HIP;
}

int hsadmm_expand(const hsadmm_plan_t* p, const float* packed, const uint8_t* mask, float* dst,
                  void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return expand_impl(p, packed, mask, dst, nullptr, nullptr, false, workspace, workspace_bytes, hip_stream);
}

int hsadmm_expand_dual(const hsadmm_plan_t* p, const float* packed, const uint8_t* mask, float* dst, const float* Zi,
                       float* Vd, void* workspace, size_t workspace_bytes, void* hip_stream)
{
    return expand_impl(p, packed, mask, dst, Zi, Vd, true, workspace, workspace_bytes, hip_stream);
}

int hsadmm_retrain_expand(const hsadmm_plan_t* p, const float* packed, const uint8_t* mask, float* dst,
                          const float* Zi, float* Vd, const float* z_prev, double* residuals, void* workspace,
                          size_t workspace_bytes, void* hip_stream)
{
    return expand_impl(p, packed, mask, dst, Zi, Vd, true, workspace, workspace_bytes, hip_stream, z_prev,
                       residuals, true);
}

const char* hsadmm_strerror(int code)
{
    switch (code) {
        case HSADMM_OK: return "ok";
        case HSADMM_ERR_INVALID_ARGUMENT: return "invalid argument";
        case HSADMM_ERR_WORKSPACE: return "workspace too small";
        case HSADMM_ERR_HIP: return "HIP runtime error";
        case HSADMM_ERR_UNSUPPORTED: return "unsupported size";
        case HSADMM_ERR_HOST_MEMORY: return "host memory allocation failed";
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
            return HSADMM_ERR_HOST_MEMORY;
        }
        for (size_t i = 0; i < 2 * kTimingPairs; ++i) {
            hipEvent_t e;
            if (hipEventCreate(&e) != hipSuccess) return HSADMM_ERR_HIP;
            p->ev.push_back(e);
        }
    }
    p->timing = enable != 0 && p->ev.size() == 2 * kTimingPairs;
    p->ev_used.store(0);
    return HSADMM_OK;
}

int hsadmm_kernel_timing_read(hsadmm_plan_t* p, double* total_ms, int64_t* launches)
{
    if (!p || !total_ms || !launches) return HSADMM_ERR_INVALID_ARGUMENT;
    for (int k = 0; k < kKernelCount; ++k) { total_ms[k] = 0.0; launches[k] = 0; }
    const size_t used = std::min(p->ev_used.load(), kTimingPairs);
    for (size_t i = 0; i < used; ++i) {
        if (hipEventSynchronize(p->ev[2 * i + 1]) != hipSuccess) return HSADMM_ERR_HIP;
        float ms = 0.f;
        if (hipEventElapsedTime(&ms, p->ev[2 * i], p->ev[2 * i + 1]) != hipSuccess) return HSADMM_ERR_HIP;
        total_ms[p->ev_kernel[i]] += (double)ms;
        launches[p->ev_kernel[i]] += 1;
    }
    p->ev_used.store(0);
    return HSADMM_OK;
}

int hsadmm_plan_estimates(const hsadmm_plan_t* p) { return (p && p->use_estimate) ? 1 : 0; }

int hsadmm_kernel_grid(const hsadmm_plan_t* p, int kernel_id)
{
    if (!p || kernel_id < 0 || kernel_id >= kKernelCount) return HSADMM_ERR_INVALID_ARGUMENT;
    return (int)p->last_grid[kernel_id].load(std::memory_order_relaxed);
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
        case kWKeys: return "weighted_pass1";
        case kWFinal: return "weighted_final";
        case kDualInter: return "dual_inter";
        case kResPart: return "residual_partials";
        case kResFinish: return "residual_finish";
        case kColsums: return "composite_colsums";
        case kChanFinal: return "channel_final";
        case kWFixup: return "weighted_fixup";
        case kBothFinal: return "composite_final";
        case kAverage: return "average";
        case kMaskDrift: return "mask_drift";
        case kFixupGather: return "fixup_gather";
        case kWFixupPack: return "weighted_fixup_pack";
        case kRetrainProject: return "retrain_project";
        case kRetrainExpand: return "retrain_expand";
        case kScaleLayers: return "scale_layers";
        case kPass1Hinted: return "project_pass1_hinted";
        case kHintedRepair: return "hinted_repair";
        case kSqnormPart: return "sqnorm_partials";
        case kResPick: return "residual_pick";
        case kWHintedRepair: return "weighted_hinted_repair";
        default: return "";
    }
}

}  // extern "C"
