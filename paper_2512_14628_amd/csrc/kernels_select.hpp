// Per-layer top-k selection (radix select on fp64 bit patterns) and the block scan it shares with scan_mask.
// Part of the single translation unit built from hsadmm.hip (included there, in order).
#ifndef KERNELS_SELECT_HPP
#define KERNELS_SELECT_HPP
#include "hsadmm_device.hpp"

namespace {

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

// Exchanges inside rows of 16 lanes, as data-parallel primitives (no LDS traffic); every lane must be active.
// After the four steps lane ^ 1, lane ^ 2, mirror inside 8 lanes, mirror inside 16 lanes, in this order, a
// lane has met every other lane of its row.
template <int CTRL>
__device__ __forceinline__ unsigned int row_exchange(unsigned int v)
{
    return (unsigned int)__builtin_amdgcn_update_dpp((int)v, (int)v, CTRL, 0xF, 0xF, false);
}
constexpr int kDppXor1 = 0xB1;          // quad_perm [1,0,3,2]
constexpr int kDppXor2 = 0x4E;          // quad_perm [2,3,0,1]
constexpr int kDppHalfMirror = 0x141;   // lane i of 8 reads lane 7 - i
constexpr int kDppMirror = 0x140;       // lane i of 16 reads lane 15 - i

__device__ __forceinline__ unsigned int lane_value(unsigned int v, int lane)   // lane: the same in every lane
{
    return (unsigned int)__builtin_amdgcn_readlane((int)v, lane);
}

// min / max over the 16 lanes of a row, in every lane of the row
__device__ __forceinline__ void row_min_max(unsigned int& mn, unsigned int& mx)
{
    unsigned int a, b;
    a = row_exchange<kDppXor1>(mn); b = row_exchange<kDppXor1>(mx); mn = a < mn ? a : mn; mx = b > mx ? b : mx;
    a = row_exchange<kDppXor2>(mn); b = row_exchange<kDppXor2>(mx); mn = a < mn ? a : mn; mx = b > mx ? b : mx;
    a = row_exchange<kDppHalfMirror>(mn); b = row_exchange<kDppHalfMirror>(mx); mn = a < mn ? a : mn; mx = b > mx ? b : mx;
    a = row_exchange<kDppMirror>(mn); b = row_exchange<kDppMirror>(mx); mn = a < mn ? a : mn; mx = b > mx ? b : mx;
}

// For lane i with value v: the sum of v over the lanes above i of the wave (`above`) and over all 64 lanes.
__device__ __forceinline__ void wave_sum_above(unsigned int v, int lane, unsigned int& above, unsigned int& total)
{
    // butterfly inside the row: at each step the two halves of a block exchange their block sums
    unsigned int tot = v, ab = 0u, p;
    p = row_exchange<kDppXor1>(tot); ab += (lane & 1) ? 0u : p; tot += p;
    p = row_exchange<kDppXor2>(tot); ab += (lane & 2) ? 0u : p; tot += p;
    p = row_exchange<kDppHalfMirror>(tot); ab += (lane & 4) ? 0u : p; tot += p;
    p = row_exchange<kDppMirror>(tot); ab += (lane & 8) ? 0u : p; tot += p;
    const unsigned int t0 = lane_value(tot, 0), t1 = lane_value(tot, 16), t2 = lane_value(tot, 32),
                       t3 = lane_value(tot, 48);
    const int row = lane >> 4;
    above = ab + (row == 0 ? t1 + t2 + t3 : row == 1 ? t2 + t3 : row == 2 ? t3 : 0u);
    total = t0 + t1 + t2 + t3;
}

constexpr int kTopkList = 32;               // candidates ranked directly instead of by further passes
struct TopkShared {
    alignas(16) unsigned int hist[3][256];     // used in turn: one fills while the next is cleared
    alignas(16) unsigned int w_lo[kScanWaves]; // per wave: smallest / largest upper key word
    alignas(16) unsigned int w_hi[kScanWaves];
    int wtot[kScanWaves];
    unsigned long long list[kTopkList];        // early exit: the few remaining candidates, in any order
    unsigned int n_list;
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
// tau, the k-th largest pattern, is found eight bits at a time on y = key - c, c = the smallest upper key
// word (lower word zero), from the most significant bit that can be set in a y downwards: one 256-bin
// histogram per pass, which every wave then reads for itself (one barrier per pass).  `need` tracks how
// many groups must still be taken from the candidates that share the prefix found so far.  Groups with
// key > tau are kept; of the groups with key == tau the first `need` in index order are kept.
// pos_l / kidx_l receive the layer's index mappings: the rank of every kept group (-1: pruned) and the
// ascending list of the kept groups.
__device__ __forceinline__ bool same_prefix(unsigned long long y, unsigned long long prefix, int known)
{
    return known >= 64 || (y >> known) == (prefix >> known);
}

template <bool INREG>
__device__ __forceinline__ void topk_layer(int G, const unsigned long long* kb, uint8_t* ml, int kk, TopkShared& sh,
                                           int32_t* pos_l, int32_t* kidx_l, int32_t* sel_l, int32_t* ck_l)
{
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    LayerKeys<INREG> keys;
    keys.load(kb, G);

    // range of the upper key words
    unsigned int lo = ~0u, hi = 0u;
    keys.for_each([&](int, unsigned long long x) {
        const unsigned int w = (unsigned int)(x >> 32);
        lo = w < lo ? w : lo;
        hi = w > hi ? w : hi;
    });
    row_min_max(lo, hi);
    {
        const unsigned int l1 = lane_value(lo, 16), l2 = lane_value(lo, 32), l3 = lane_value(lo, 48);
        const unsigned int h1 = lane_value(hi, 16), h2 = lane_value(hi, 32), h3 = lane_value(hi, 48);
        lo = lo < l1 ? lo : l1; lo = lo < l2 ? lo : l2; lo = lo < l3 ? lo : l3;   // complete in row 0
        hi = hi > h1 ? hi : h1; hi = hi > h2 ? hi : h2; hi = hi > h3 ? hi : h3;
    }
    if (lane == 0) { sh.w_lo[wave] = lo; sh.w_hi[wave] = hi; }
    if (tid < 768) (&sh.hist[0][0])[tid] = 0u;
    if (tid == 768) sh.n_list = 0u;
    __syncthreads();
    lo = sh.w_lo[lane & (kScanWaves - 1)];
    hi = sh.w_hi[lane & (kScanWaves - 1)];
    static_assert(kScanWaves == 16, "one row of lanes holds one value per wave");
    row_min_max(lo, hi);
    const unsigned long long c = (unsigned long long)lo << 32;
    const unsigned int span = hi - lo;                        // every y is below (span + 1) << 32

    const int top = span ? 63 - __clz((int)span) : 31;        // no y has a bit above this one
    int shift = top - 7;                                      // the first digit ends at that bit
    int known = top + 1;                                      // bits >= known of y agree with the prefix so far
    unsigned long long prefix = 0ull;
    unsigned int need_now = (unsigned int)kk, cand = (unsigned int)G;
    int pass = 0;
    for (;;) {
        unsigned int* h = sh.hist[pass % 3];
        keys.for_each([&](int, unsigned long long x) {
            const unsigned long long y = x - c;
            if (same_prefix(y, prefix, known)) atomicAdd(&h[(unsigned int)(y >> shift) & 255u], 1u);
        });
        if (tid < 256) sh.hist[(pass + 1) % 3][tid] = 0u;      // last read two barriers ago
        __syncthreads();
        // every wave for itself: lane i owns bins 4i..4i+3; `above` = number of candidates in higher bins
        const uint4 hv = *reinterpret_cast<const uint4*>(&h[4 * lane]);
        const unsigned int hh[4] = {hv.x, hv.y, hv.z, hv.w};
        unsigned int above, all;
        wave_sum_above(hv.x + hv.y + hv.z + hv.w, lane, above, all);
        unsigned int bin = 0u, need_next = 0u, cand_next = 0u;
        bool mine = false;
#pragma unroll
        for (int b = 3; b >= 0; --b) {
            if (above < need_now && need_now <= above + hh[b]) {
                mine = true;
                bin = (unsigned int)(4 * lane + b);
                need_next = need_now - above;
                cand_next = hh[b];
            }
            above += hh[b];
        }
        const unsigned long long owners = __ballot(mine);      // one lane, as 1 <= need <= number of candidates
        const int owner = owners ? __builtin_ctzll(owners) : 0;
        bin = lane_value(bin, owner);
        need_now = lane_value(need_next, owner);
        cand = lane_value(cand_next, owner);
        // a digit that reaches below bit 0 of the previous one repeats bits the prefix already has
        prefix |= (unsigned long long)bin << shift;
        ++pass;
        known = shift;
        if (shift == 0 || cand <= (unsigned int)kTopkList) break;
        shift = shift > 8 ? shift - 8 : 0;
    }
    unsigned long long tau;
    int need;
    bool scan_ties;
    if (known > 0) {
        // few candidates left before the last bit: list them, then every wave ranks them directly
        keys.for_each([&](int, unsigned long long x) {
            if (same_prefix(x - c, prefix, known)) {
                const unsigned int j = atomicAdd(&sh.n_list, 1u);
                if (j < (unsigned int)kTopkList) sh.list[j] = x;
            }
        });
        __syncthreads();
        const int n = (int)cand;
        const unsigned long long mine = lane < n ? sh.list[lane] : 0ull;
        unsigned int gt = 0u, eq = 0u;          // candidates above / equal to this lane's
        for (int j = 0; j < n; ++j) {
            const unsigned long long v = sh.list[j];
            gt += v > mine ? 1u : 0u;
            eq += v == mine ? 1u : 0u;
        }
        // tau is the need_now-th largest candidate
        const unsigned long long owners = __ballot(lane < n && gt < need_now && need_now <= gt + eq);
        const int owner = owners ? __builtin_ctzll(owners) : 0;
        tau = ((unsigned long long)lane_value((unsigned int)(mine >> 32), owner) << 32) |
              (unsigned long long)lane_value((unsigned int)mine, owner);
        need = (int)(need_now - lane_value(gt, owner));
        scan_ties = (unsigned int)need != lane_value(eq, owner);   // fewer wanted than tied: index order decides
    } else {
        tau = prefix + c;
        need = (int)need_now;
        scan_ties = need_now != cand;                          // fewer wanted than tied: index order decides
    }
    // final pass in index order: the kept flag (ties: the first `need` groups equal to tau), then the rank
    // of every kept group among the kept ones
    int carry_eq = 0, carry_kept = 0;
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
        bool kept = (g < G) && (x >= tau);
        if (scan_ties) {
            const bool eq = (g < G) && (x == tau);
            const bool gt = (g < G) && (x > tau);
            int total;
            const int rank = carry_eq + block_excl_scan<kScanWaves>(eq, sh.wtot, total);
            kept = gt || (eq && rank < need);
            carry_eq += total;
        }
        int total_kept;
        const int r = carry_kept + block_excl_scan<kScanWaves>(kept, sh.wtot, total_kept);
        if (g < G) {
            ml[g] = kept ? 1 : 0;
            pos_l[g] = kept ? r : -1;
            if (sel_l) sel_l[g] = kept ? r : -1;
            if (kept) kidx_l[r] = g;
            if (kept && ck_l) ck_l[r] = g;
        }
        carry_kept += total_kept;
    }
}

// After a FILTER layer's selection under a prediction: the layer's row items that the repair pass has to visit are
// appended to the work list.  A row needs a visit unless its prediction was right and left it in final form:
// predicted kept and kept (with a compaction: at the same rank), or predicted pruned and pruned.  (This list is
// used when the dual is written out of place; updated in place, every pruned row still has to be cleared and the
// repair pass visits all items.)  Every thread looks at the rows tid, tid + 1024, ... and marks the item a row in
// need belongs to in `bits`; the marked items are then appended in index order.  The repair pass looks at every
// row of a listed item again, so listing too much is harmless: a layer with more items than `bits` holds is
// listed whole.
constexpr int kItemBits = 3 * 256 * 32;
__device__ __forceinline__ void list_repairs(const DevLayer& L, const WorkList& wl, const WorkItem* __restrict__ row_items,
                                             const int32_t* pos_l, unsigned int* bits, int* wtot, int* slot)
{
    const int tid = threadIdx.x;
    const int32_t* hp_l = wl.sel_prev + L.group_base;
    const int rows_per_item = row_items[L.rows_item0].nr;        // every item of a layer but the last has this many
    const bool all = L.rows_items > kItemBits;
    __syncthreads();                                             // the ranks written above are visible to the workgroup
    if (!all) {
        for (int w = tid; w < (L.rows_items + 31) / 32; w += kScanBlock) bits[w] = 0u;
        __syncthreads();
        for (int r = tid; r < L.c_out; r += kScanBlock) {
            const int hp = hp_l[r], pn = pos_l[r];
            const bool pred_kept = hp >= 0, kept = pn >= 0;
            const bool needs = pred_kept != kept || (kept && wl.pack && pn != hp);
            if (needs) {
                const int i = r / rows_per_item;
                atomicOr(&bits[i >> 5], 1u << (i & 31));
            }
        }
        __syncthreads();
    }
    for (int base = 0; base < L.rows_items; base += kScanBlock) {
        const int i = base + tid;
        const bool needs = i < L.rows_items && (all || ((bits[i >> 5] >> (i & 31)) & 1u) != 0u);
        int total;
        const int rank = block_excl_scan<kScanWaves>(needs, wtot, total);
        if (tid == 0 && total > 0) *slot = atomicAdd(wl.work, total);
        __syncthreads();
        if (needs) wl.work[kWorkHeader + *slot + rank] = L.rows_item0 + i;
    }
}

// After a CHANNEL layer's selection under a prediction (dual out of place): pass 1 has written the layer in the form
// the predicted channels make final.  If the selection differs from the prediction in any channel (with a
// compaction: or in any rank, which only a record that no selection of this plan wrote can cause), every row item
// of the layer is listed and the repair pass forms the layer again.  The same after the second selection of a layer
// under both constraints, over its filters and its channels (pos_l: the ranks of the layer's first group on).
__device__ __forceinline__ void list_changed_layer(const DevLayer& L, const WorkList& wl, const int32_t* pos_l, int* slot)
{
    const int tid = threadIdx.x;
    const int32_t* hp_l = wl.sel_prev + L.group_base;
    __syncthreads();                                             // the ranks written above are visible to the workgroup
    bool differs = false;
    for (int g = tid; g < L.G; g += kScanBlock) {
        const int hp = hp_l[g], pn = pos_l[g];
        const bool pred_kept = hp >= 0, kept = pn >= 0;
        differs = differs || pred_kept != kept || (kept && wl.pack && pn != hp);
    }
    if (!__syncthreads_or(differs)) return;
    if (tid == 0) *slot = atomicAdd(wl.work, L.rows_items);
    __syncthreads();
    for (int i = tid; i < L.rows_items; i += kScanBlock) wl.work[kWorkHeader + *slot + i] = L.rows_item0 + i;
}

// Rows 0 and 1 of the residual norms of a FILTER or unconstrained layer whose pass 1 took, per group, the sums of
// either outcome: rowres[4g + 0, 2] if group g is kept, rowres[4g + 1, 3] if it is pruned.  Thread t adds the groups
// t, t + 1024, ... in order; threads are combined by a butterfly per wave and the waves in order: a fixed order.
__device__ __forceinline__ void pick_residuals(const DevLayer& L, int l, int n_layers, const uint8_t* ml,
                                               const WorkList& wl, double (*red)[2])
{
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = tid / kWave;
    __syncthreads();                                             // the mask written above is visible to the workgroup
    double s0 = 0.0, s1 = 0.0;
    for (int g = tid; g < L.G; g += kScanBlock) {
        const bool kept = ml[g] != 0;
        const double* r = wl.rowres + 4 * (int64_t)(L.group_base + g);
        s0 += kept ? r[0] : r[1];
        s1 += kept ? r[2] : r[3];
    }
    s0 = wave_xor_sum(s0, kWave);
    s1 = wave_xor_sum(s1, kWave);
    if (lane == 0) { red[wave][0] = s0; red[wave][1] = s1; }
    __syncthreads();
    if (tid < 2) {
        double t = red[0][tid];
        for (int w = 1; w < kScanWaves; ++w) t += red[w][tid];
        wl.res_out[(int64_t)tid * n_layers + l] = t;
    }
}

// One workgroup per layer: finish the CHANNEL keys, then write the layer's mask.
// stage 0: workgroup b takes layer b; of a BOTH layer it selects the filters (its first c_out groups).
// stage 1: workgroup b takes layer layer_list[b], a BOTH layer, and selects its channels (the c_in
//          groups after the filters) from the column sums composite_colsums left in colpart.
// out[j] = sum over the row blocks (ascending) of part[rb * row_len + j] for the columns j < ncols: a thread takes
// the columns tid, tid + 1024, ..., four of them at a time and four row blocks each (sixteen loads in flight).
constexpr int kColChunk = 4096;             // columns of the channel keys' LDS staging
__device__ __forceinline__ void sum_rowblocks(const double* __restrict__ part, int ncols, int row_len, int n_rowblocks,
                                              double* out)
{
    for (int j0 = threadIdx.x; j0 < ncols; j0 += 4 * kScanBlock) {
        const int nc = (ncols - j0 + kScanBlock - 1) / kScanBlock;           // columns of this round (4 or fewer)
        const double* c0 = part + j0;
        double acc[4] = {0.0, 0.0, 0.0, 0.0};
        int rb = 0;
        for (; rb + 4 <= n_rowblocks; rb += 4) {
            double x[4][4];
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int b = 0; b < 4; ++b)
                    x[c][b] = (c < nc) ? c0[c * kScanBlock + (int64_t)(rb + b) * row_len] : 0.0;
#pragma unroll
            for (int c = 0; c < 4; ++c)
#pragma unroll
                for (int b = 0; b < 4; ++b) acc[c] += x[c][b];
        }
        for (; rb < n_rowblocks; ++rb)
#pragma unroll
            for (int c = 0; c < 4; ++c)
                if (c < nc) acc[c] += c0[c * kScanBlock + (int64_t)rb * row_len];
#pragma unroll
        for (int c = 0; c < 4; ++c)
            if (c < nc) out[j0 + c * kScanBlock] = acc[c];
    }
}

// NEST: the plan has layers whose channels come in runs (a kernel of its own, so that plans without such layers run
// the plain selection unchanged).
template <bool NEST>
__global__ __launch_bounds__(kScanBlock) void select_topk(const DevLayer* __restrict__ layers,
                                                          double* __restrict__ key,
                                                          const double* __restrict__ colpart,
                                                          uint8_t* __restrict__ mask,
                                                          const int32_t* __restrict__ layer_list, int stage,
                                                          IndexMaps im, int n_layers, int pack_align,
                                                          WorkList wl, const WorkItem* __restrict__ row_items,
                                                          unsigned char* __restrict__ nest)
{
    __shared__ TopkShared sh;
    __shared__ double colsum[kColChunk];
    __shared__ int work_slot;
    __shared__ double res_red[kScanWaves][2];
    const DevLayer L = layers[stage == 0 ? (int)blockIdx.x : layer_list[blockIdx.x]];
    const bool both = L.mode == HSADMM_MODE_BOTH;
    const bool channels = L.mode == HSADMM_MODE_CHANNEL || (both && stage == 1);
    const int G = both ? (stage == 0 ? L.c_out : L.c_in) : L.G;
    const int first = L.group_base + ((both && stage == 1) ? L.c_out : 0);
    const int tid = threadIdx.x;
    double* kl = key + first;
    uint8_t* ml = mask + first;
    // the index mappings of this selection (what scan_mask would derive from the mask)
    int32_t* pos_l = im.pos + first;
    int32_t* sel_l = im.sel ? im.sel + first : nullptr;      // the caller's copy of the ranks
    int32_t* kidx_l = im.kept_idx + L.kept_start + ((both && stage == 1) ? L.k : 0);
    int32_t* ck_l = wl.co.kept_idx ? wl.co.kept_idx + (kidx_l - im.kept_idx) : nullptr;   // the caller's copy of the kept list
    if (tid == 0 && stage == 0 && wl.co.layer_off) {
        const int l = blockIdx.x;
        wl.co.layer_off[l] = L.packed_off;
        if (l == n_layers - 1)
            wl.co.layer_off[n_layers] = L.packed_off + packed_size(L.mode, L.unit, (L.mode == HSADMM_MODE_NONE) ? L.G : L.k,
                                                                   L.k_in, pack_align);
    }
    if (tid == 0 && stage == 0) {
        const int l = blockIdx.x;
        const int c0 = (L.mode == HSADMM_MODE_NONE) ? L.G : L.k;
        im.cnt[l] = c0;
        im.cnt[n_layers + l] = L.kept_start;
        im.cnt[2 * n_layers + l] = both ? L.k_in : 0;
        im.layer_off[l] = L.packed_off;
        if (l == n_layers - 1) im.layer_off[n_layers] = L.packed_off + packed_size(L.mode, L.unit, c0, L.k_in, pack_align);
    }
    if (channels) {
        // key[c]: every column of the channel summed over the row blocks (ascending), then the channel's khw column
        // sums added (ascending); the same order for every channel of a layer, wherever it lies
        const double* cp = colpart + L.colpart_off;
        if (L.khw == 1 && G > kScanBlock) {
            sum_rowblocks(cp, G, L.row_len, L.n_rowblocks, kl);
        } else if (L.khw > 1 && L.khw <= kColChunk) {
            // the columns of the view first (coalesced: a thread per column, as above), a chunk of whole channels at
            // a time into LDS, then every channel's khw column sums in ascending order
            const int chunk_ch = kColChunk / L.khw;
            for (int ch0 = 0; ch0 < G; ch0 += chunk_ch) {
                const int nch = min(chunk_ch, G - ch0);
                sum_rowblocks(cp + (int64_t)ch0 * L.khw, nch * L.khw, L.row_len, L.n_rowblocks, colsum);
                __syncthreads();
                for (int g = tid; g < nch; g += kScanBlock) {
                    double acc = 0.0;
                    for (int t = 0; t < L.khw; ++t) acc += colsum[g * L.khw + t];
                    kl[ch0 + g] = acc;
                }
                __syncthreads();
            }
        } else
        for (int g = tid; g < G; g += kScanBlock) {
            double acc = 0.0;
            const double* cg = cp + (int64_t)g * L.khw;
            int rb = 0;
            // same order of additions as the plain loop below, with many loads in flight
            if (L.khw == 1) {
                for (; rb + 16 <= L.n_rowblocks; rb += 16) {
                    double x[16];
#pragma unroll
                    for (int b = 0; b < 16; ++b) x[b] = cg[(int64_t)(rb + b) * L.row_len];
#pragma unroll
                    for (int b = 0; b < 16; ++b) acc += x[b];
                }
            }
            for (; rb < L.n_rowblocks; ++rb)
                for (int t = 0; t < L.khw; ++t) acc += cg[(int64_t)rb * L.row_len + t];
            kl[g] = acc;
        }
        __syncthreads();
    }
    const int kk = (L.mode == HSADMM_MODE_NONE) ? G : ((both && stage == 1) ? L.k_in : L.k);
    const unsigned long long* kb = reinterpret_cast<const unsigned long long*>(kl);
    // Channels that come in runs of `span` (shape groups inside input channels, Section 2.1): first the runs are
    // ranked by the sum of their channels' keys and k_coarse of them stay; then the channels of those runs alone are
    // ranked.  The second ranking sees key pattern + 1 for a channel of a kept run and 0 for any other, so no channel
    // of a pruned run can be taken, whatever ties at zero there are; such a channel's key is reported as 0, the norm
    // it has once its run is pruned.
    const bool nested = NEST && channels && L.span >= 1;
    const int C = nested ? G / L.span : 0;
    double* run_key = nested ? reinterpret_cast<double*>(nest + L.nest_off) : nullptr;
    unsigned long long* shifted = reinterpret_cast<unsigned long long*>(run_key + C);
    int32_t* run_pos = reinterpret_cast<int32_t*>(shifted + G);
    int32_t* run_kidx = run_pos + C;
    uint8_t* run_mask = reinterpret_cast<uint8_t*>(run_kidx + C);
    if (nested) {
        for (int j = tid; j < C; j += kScanBlock) {
            double acc = 0.0;
            for (int t = 0; t < L.span; ++t) acc += kl[(int64_t)j * L.span + t];
            run_key[j] = acc;
        }
        __syncthreads();
    }
    if constexpr (!NEST) {
        if (kk >= G) {
            for (int g = tid; g < G; g += kScanBlock) {
                ml[g] = 1; pos_l[g] = g; kidx_l[g] = g;
                if (sel_l) sel_l[g] = g;
                if (ck_l) ck_l[g] = g;
            }
        } else if (G <= kTopkRegs * kScanBlock) {
            topk_layer<true>(G, kb, ml, kk, sh, pos_l, kidx_l, sel_l, ck_l);
        } else {
            topk_layer<false>(G, kb, ml, kk, sh, pos_l, kidx_l, sel_l, ck_l);
        }
    } else
    for (int phase = nested ? 0 : 1; phase < 2; ++phase) {
        const bool runs = phase == 0;
        const int Gp = runs ? C : G;
        const int kp = runs ? L.k_coarse : kk;
        const unsigned long long* kbp = runs ? reinterpret_cast<const unsigned long long*>(run_key) : kb;
        uint8_t* mlp = runs ? run_mask : ml;
        int32_t* posp = runs ? run_pos : pos_l;
        int32_t* kidxp = runs ? run_kidx : kidx_l;
        int32_t* selp = runs ? nullptr : sel_l;
        int32_t* ckp = runs ? nullptr : ck_l;
        if (kp >= Gp) {
            for (int g = tid; g < Gp; g += kScanBlock) {
                mlp[g] = 1; posp[g] = g; kidxp[g] = g;
                if (selp) selp[g] = g;
                if (ckp) ckp[g] = g;
            }
        } else if (Gp <= kTopkRegs * kScanBlock) {
            topk_layer<true>(Gp, kbp, mlp, kp, sh, posp, kidxp, selp, ckp);
        } else {
            topk_layer<false>(Gp, kbp, mlp, kp, sh, posp, kidxp, selp, ckp);
        }
        if (runs) {
            __syncthreads();                                 // the runs' mask is complete
            for (int g = tid; g < G; g += kScanBlock) {
                const bool in = run_mask[g / L.span] != 0;
                shifted[g] = in ? kb[g] + 1ull : 0ull;
                if (!in) kl[g] = 0.0;
            }
            __syncthreads();
            kb = shifted;
        }
    }
    if (wl.res_out && stage == 0 && (L.mode == HSADMM_MODE_FILTER || L.mode == HSADMM_MODE_NONE))
        pick_residuals(L, (int)blockIdx.x, n_layers, ml, wl, res_red);
    if (wl.sel_prev && L.mode == HSADMM_MODE_FILTER)
        list_repairs(L, wl, row_items, pos_l, &sh.hist[0][0], sh.wtot, &work_slot);
    else if (wl.sel_prev && wl.channels && L.mode == HSADMM_MODE_CHANNEL)
        list_changed_layer(L, wl, pos_l, &work_slot);
    else if (wl.sel_prev && wl.both && both && stage == 1)
        list_changed_layer(L, wl, im.pos + L.group_base, &work_slot);       // filters (an earlier launch) and channels
}

}  // namespace
#endif
