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
// pos_l / kidx_l receive the layer's index mappings: the rank of every kept group (-1: pruned) and the
// ascending list of the kept groups.
template <bool INREG>
__device__ __forceinline__ void topk_layer(int G, const unsigned long long* kb, uint8_t* ml, int kk, TopkShared& sh,
                                           int32_t* pos_l, int32_t* kidx_l)
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
            if (kept) kidx_l[r] = g;
        }
        carry_kept += total_kept;
    }
}

// One workgroup per layer: finish the CHANNEL keys, then write the layer's mask.
// stage 0: workgroup b takes layer b; of a BOTH layer it selects the filters (its first c_out groups).
// stage 1: workgroup b takes layer layer_list[b], a BOTH layer, and selects its channels (the c_in
//          groups after the filters) from the column sums composite_colsums left in colpart.
__global__ __launch_bounds__(kScanBlock) void select_topk(const DevLayer* __restrict__ layers,
                                                          double* __restrict__ key,
                                                          const double* __restrict__ colpart,
                                                          uint8_t* __restrict__ mask,
                                                          const int32_t* __restrict__ layer_list, int stage,
                                                          IndexMaps im, int n_layers, int pack_align)
{
    __shared__ TopkShared sh;
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
    int32_t* kidx_l = im.kept_idx + L.kept_start + ((both && stage == 1) ? L.k : 0);
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
        // key[c] = sum over row blocks (ascending), then over the channel's khw columns (ascending)
        const double* cp = colpart + L.colpart_off;
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
            if (L.khw <= 9) {
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
    const int kk = (L.mode == HSADMM_MODE_NONE) ? G : ((both && stage == 1) ? L.k_in : L.k);
    if (kk >= G) {
        for (int g = tid; g < G; g += kScanBlock) { ml[g] = 1; pos_l[g] = g; kidx_l[g] = g; }
        return;
    }
    const unsigned long long* kb = reinterpret_cast<const unsigned long long*>(kl);
    if (G <= kTopkRegs * kScanBlock) topk_layer<true>(G, kb, ml, kk, sh, pos_l, kidx_l);
    else topk_layer<false>(G, kb, ml, kk, sh, pos_l, kidx_l);
}

}  // namespace
#endif
