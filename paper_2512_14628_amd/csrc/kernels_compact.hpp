// hsadmm_compact / hsadmm_expand: mask scan, gather into the packed buffer, zero fill + scatter back.
// Part of the single translation unit built from hsadmm.hip (included there, in order).
#ifndef KERNELS_COMPACT_HPP
#define KERNELS_COMPACT_HPP
#include "hsadmm_device.hpp"
#include "kernels_select.hpp"

namespace {

// ------------------------------------------------------------------ mask scan (compact / expand)

__device__ __forceinline__ int nonzero_bytes(unsigned int x)
{
    // bit 7 of every byte becomes 1 iff the byte is nonzero
    const unsigned int t = (((x & 0x7f7f7f7fu) + 0x7f7f7f7fu) | x) & 0x80808080u;
    return __popc(t);
}

// One workgroup per layer.  The groups of a layer form one scan segment (a BOTH layer two: its
// filters, then its channels).  Every workgroup counts the kept groups of all segments in one flat
// pass over the mask, 16 groups per thread and step: chunk_layer gives the segment of a 16-group
// chunk that lies inside one constrained segment (one 128-bit load, a popcount, and one LDS add per
// wave when the whole wave sits in one segment); chunks that straddle segments or touch an
// unconstrained layer (0xffff) go group by group through group_layer (bit 15 marks an unconstrained
// layer, whose groups are always kept).  The workgroup then sums the aligned packed sizes of layers
// 0..l-1 to get its own offset in the packed buffer and scans its own layer's mask.  Packed starts
// are multiples of pack_align, so the offset is the plain sum of the rounded-up sizes.
__global__ __launch_bounds__(kScanBlock) void scan_mask(const DevLayer* __restrict__ layers, int nL, int nSeg,
                                                        int n_groups, int pack_align,
                                                        const uint8_t* __restrict__ mask,
                                                        const uint16_t* __restrict__ group_layer,
                                                        const uint16_t* __restrict__ chunk_layer, IndexMaps o)
{
    __shared__ int cnt[2 * HSADMM_MAX_LAYERS];      // per segment
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
    int mode_j = 0, seg_j = 0;
    if (tid < l) { unit_j = layers[tid].unit; mode_j = layers[tid].mode; seg_j = layers[tid].seg0; }
    for (int j = tid; j < nSeg; j += kScanBlock) cnt[j] = 0;
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
        const int c0 = cnt[seg_j];
        const int c1 = (mode_j == HSADMM_MODE_BOTH) ? cnt[seg_j + 1] : 0;
        sz = packed_size(mode_j, unit_j, c0, c1, pack_align);
        kept_before = c0 + c1;
    }
    for (int j = tid + kScanBlock; j < l; j += kScanBlock) {    // more than 1024 layers
        const int mj = layers[j].mode, sj = layers[j].seg0;
        const int c0 = cnt[sj];
        const int c1 = (mj == HSADMM_MODE_BOTH) ? cnt[sj + 1] : 0;
        sz += packed_size(mj, layers[j].unit, c0, c1, pack_align);
        kept_before += c0 + c1;
    }
    sz = wave_sum_i64(sz);
    kept_before = wave_sum_i32(kept_before);
    if (lane == 0) { wsum[wave] = sz; wkept[wave] = kept_before; }
    __syncthreads();
    long long pos = 0;
    int kb = 0;
#pragma unroll
    for (int w = 0; w < kScanWaves; ++w) { pos += wsum[w]; kb += wkept[w]; }
    const bool both = L.mode == HSADMM_MODE_BOTH;
    const int own0 = cnt[L.seg0];
    const int own1 = both ? cnt[L.seg0 + 1] : 0;
    if (tid == 0) {
        o.layer_off[l] = pos;
        o.cnt[l] = own0;
        o.cnt[nL + l] = kb;
        o.cnt[2 * nL + l] = own1;
        if (l == nL - 1) {
            const long long s = packed_size(L.mode, L.unit, own0, own1, pack_align);
            o.layer_off[nL] = pos + s;
        }
    }
    // ranks inside each of the layer's segments; kept_idx lists the first segment, then the second
    for (int seg = 0; seg < (both ? 2 : 1); ++seg) {
        const int G = both ? (seg == 0 ? L.c_out : L.c_in) : L.G;
        const int g_first = L.group_base + (seg == 1 ? L.c_out : 0);
        const int k_first = kb + (seg == 1 ? own0 : 0);
        int carry = 0;
        for (int base = 0; base < G; base += kScanBlock) {
            const int g = base + tid;
            const bool m = (g < G) && (L.mode == HSADMM_MODE_NONE || mask[g_first + g] != 0);
            int total;
            const int rank = carry + block_excl_scan<kScanWaves>(m, wtot, total);
            if (g < G) {
                o.pos[g_first + g] = m ? rank : -1;
                if (o.sel) o.sel[g_first + g] = m ? rank : -1;
                if (m) o.kept_idx[k_first + rank] = g;
            }
            carry += total;
        }
    }
}

// ------------------------------------------------------------------ compaction (gather)

// SUM: the source is the element-wise sum of two arenas (c = z_i + v_i, Section 4.4.1), formed on the fly.
template <bool SUM>
__device__ __forceinline__ void gather_item(const WorkItem& it, const float* src, const float* src1,
                                            const int32_t* __restrict__ pos, const int32_t* __restrict__ cnt,
                                            const int32_t* __restrict__ kept_idx, int n_layers,
                                            const int64_t* __restrict__ layer_off, float* packed, CopyOut co)
{
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = it.row_len;
    if (it.row0 == 0) copy_out_layer(it.layer, cnt, kept_idx, n_layers, layer_off, co);
    float* out = packed + layer_off[it.layer];
    if (!mode_has_channels(item_mode(it))) {
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
        // j = q*khw + t comes from source column kept[q]*khw + t.  it.row0 is the index of the item's
        // first row inside the layer.  A wave takes a row; a lane gathers 4 adjacent packed columns
        // and stores them with one 128-bit access.  BOTH: only the kept filters' rows are packed, at
        // their rank among the kept filters; the kept channels follow the kept filters in kept_idx.
        const bool both = item_mode(it) == HSADMM_MODE_BOTH;
        const int kc = both ? cnt[2 * n_layers + it.layer] : cnt[it.layer];
        const int khw = it.khw;
        const int out_len = kc * khw;
        const int32_t* kl = kept_idx + cnt[n_layers + it.layer] + (both ? cnt[it.layer] : 0);
        const DivKhw div(khw);
        const int quads = out_len >> 2;
        constexpr int kRows = 2;      // rows a wave keeps in flight: their loads are issued together
        const WaveShare ws(it.nr, wave);
        for (int rr0 = ws.row; rr0 < it.nr; rr0 += kRows * ws.rows_at_once) {
            int prow[kRows];
            int64_t ro[kRows];
#pragma unroll
            for (int u = 0; u < kRows; ++u) {
                const int rr = rr0 + u * ws.rows_at_once;
                prow[u] = -1;
                if (rr < it.nr) prow[u] = both ? pos[it.g0 + rr] : it.row0 + rr;
                ro[u] = it.base + (int64_t)rr * row_len;
            }
            auto at = [&](int u, int idx) -> float {
                return SUM ? ld1(src + ro[u] + idx) + ld1(src1 + ro[u] + idx) : ld1(src + ro[u] + idx);
            };
            for (int j4 = lane + ws.first; j4 < quads; j4 += ws.stride) {
                const int j = j4 << 2;
                int4 c;
                if (khw == 1) {
                    __builtin_memcpy(&c, kl + j, 16);
                } else {
                    const int q0 = div(j), q1 = div(j + 1), q2 = div(j + 2), q3 = div(j + 3);
                    c.x = kl[q0] * khw + (j - q0 * khw);
                    c.y = kl[q1] * khw + (j + 1 - q1 * khw);
                    c.z = kl[q2] * khw + (j + 2 - q2 * khw);
                    c.w = kl[q3] * khw + (j + 3 - q3 * khw);
                }
                v4f v[kRows];
#pragma unroll
                for (int u = 0; u < kRows; ++u) {
                    if (prow[u] < 0) continue;
                    v[u].x = at(u, c.x); v[u].y = at(u, c.y); v[u].z = at(u, c.z); v[u].w = at(u, c.w);
                }
#pragma unroll
                for (int u = 0; u < kRows; ++u)
                    if (prow[u] >= 0) st4u(out + (int64_t)prow[u] * out_len + j, v[u]);
            }
            for (int j = (quads << 2) + lane + ws.first; j < out_len; j += ws.stride) {
                const int q = div(j);
                const int cs = kl[q] * khw + (j - q * khw);
#pragma unroll
                for (int u = 0; u < kRows; ++u)
                    if (prow[u] >= 0) out[(int64_t)prow[u] * out_len + j] = at(u, cs);
            }
        }
    }
}

template <bool SUM>
__global__ __launch_bounds__(kBlock) void compact_gather(const WorkItem* __restrict__ items,
                                                         const float* __restrict__ src,
                                                         const float* __restrict__ src1,
                                                         const int32_t* __restrict__ pos,
                                                         const int32_t* __restrict__ cnt,
                                                         const int32_t* __restrict__ kept_idx, int n_layers,
                                                         const int64_t* __restrict__ layer_off,
                                                         float* __restrict__ packed, CopyOut co)
{
    gather_item<SUM>(items[blockIdx.x], src, src1, pos, cnt, kept_idx, n_layers, layer_off, packed, co);
}

// The FILTER fix-up and the compaction of Z in one launch: the fix-up rewrites pruned rows only, the gather
// reads kept rows only (final since pass 1), so the two kinds of workgroup touch disjoint memory and need no
// order between them.  Workgroups [0, n_fix) take the fix-up items, the rest the row items.
__global__ __launch_bounds__(kBlock) void fixup_gather(const WorkItem* __restrict__ fix_items, int n_fix,
                                                       const uint8_t* __restrict__ mask, float* U, float* Z,
                                                       const WorkItem* __restrict__ row_items,
                                                       const int32_t* __restrict__ pos,
                                                       const int32_t* __restrict__ cnt,
                                                       const int32_t* __restrict__ kept_idx, int n_layers,
                                                       const int64_t* __restrict__ layer_off, float* packed,
                                                       CopyOut co)
{
    if ((int)blockIdx.x < n_fix)
        fixup_rows(fix_items[blockIdx.x], mask, U, Z);
    else
        gather_item<false>(row_items[(int)blockIdx.x - n_fix], Z, nullptr, pos, cnt, kept_idx, n_layers, layer_off,
                           packed, co);
}

// After the selection of a step whose pass 1 formed its own prediction (kernels_estimate.hpp): every FILTER row from
// the form pass 1 gave it (pred, a prediction record without ranks) to its final form (hinted_repair_rows with the
// dual in place).  project_fixup_est: the projection alone.  fixup_gather_est: with a compaction, kept rows are packed
// on the way and the rows of the unconstrained layers gathered in the same launch; workgroups [0, n_fix) take the
// FILTER row items, the rest those of the unconstrained layers.
template <int R>
__global__ __launch_bounds__(kBlock) void project_fixup_est(const WorkItem* __restrict__ fix_items, ProjectArgs a, int Rrt,
                                                            const int32_t* __restrict__ pred,
                                                            const int32_t* __restrict__ pos)
{
    hinted_repair_rows<R>(fix_items[blockIdx.x], a, Rrt, pred, pos, true, nullptr);
}

template <int R>
__global__ __launch_bounds__(kBlock) void fixup_gather_est(const WorkItem* __restrict__ fix_items, int n_fix,
                                                           ProjectArgs a, int Rrt, const int32_t* __restrict__ pred,
                                                           const WorkItem* __restrict__ none_items, PackOut po)
{
    if ((int)blockIdx.x < n_fix) {
        const WorkItem it = fix_items[blockIdx.x];
        hinted_repair_rows<R>(it, a, Rrt, pred, po.pos, true, po.packed + it.packed_off);
    } else {
        gather_item<false>(none_items[(int)blockIdx.x - n_fix], a.Z, nullptr, po.pos, po.cnt, po.kept_idx, po.n_layers,
                           po.layer_off, po.packed, po.co);
    }
}

// The final pass of CHANNEL or BOTH layers with its packing (project_frozen<R, true>) and the gather of the plain
// layers' rows (FILTER / NONE, final before this launch) in one launch: workgroups [0, n_final) take the final-pass
// items, the rest the plain row items.  The two kinds of workgroup touch different layers.
template <int R>
__global__ __launch_bounds__(kBlock) void final_gather(const WorkItem* __restrict__ final_items, int n_final,
                                                       ProjectArgs a, int Rrt, const uint8_t* __restrict__ mask,
                                                       PackOut po, const WorkItem* __restrict__ plain_items)
{
    if ((int)blockIdx.x < n_final)
        frozen_item<R, true>(final_items[blockIdx.x], a, Rrt, mask, po);
    else
        gather_item<false>(plain_items[(int)blockIdx.x - n_final], a.Z, nullptr, po.pos, po.cnt, po.kept_idx,
                           po.n_layers, po.layer_off, po.packed, po.co);
}

// The weighted FILTER fix-up with its kept rows packed as they are formed, and the compaction c = Z + Vd of the
// other layers' rows (final before this launch), in one launch: workgroups [0, n_fix) take the fix-up items, the
// rest the row items of the layers that are not FILTER layers.
__global__ __launch_bounds__(kBlock) void weighted_fixup_pack(const WorkItem* __restrict__ fix_items, int n_fix,
                                                              const uint8_t* __restrict__ mask, float* U, float* Z,
                                                              const float* __restrict__ Zg, const float* Vd,
                                                              const float* __restrict__ coef,
                                                              const WorkItem* __restrict__ rest_items, PackOut po)
{
    if ((int)blockIdx.x < n_fix)
        weighted_fixup_rows<true>(fix_items[blockIdx.x], mask, U, Z, Zg, Vd, coef, po);
    else
        gather_item<true>(rest_items[(int)blockIdx.x - n_fix], Z, Vd, po.pos, po.cnt, po.kept_idx, po.n_layers,
                          po.layer_off, po.packed, po.co);
}

// ------------------------------------------------------------------ expansion (zero fill + scatter)

// DUAL: the expanded tensor is the new global consensus z, and the inter-node dual update of Eq. (13),
// Vd <- Vd + (Zi - z), is applied in the same pass (z is not read back from memory).
// RES (with DUAL): the item's inter-node residual sums of Section 3.4, (Zi - z)^2 and (z - z_prev)^2 in fp64,
// also go to part[4 * item + 2, 3]; z_prev is a buffer other than dst.
template <bool DUAL, bool RES = false>
__global__ __launch_bounds__(kBlock) void expand_scatter(const WorkItem* __restrict__ items,
                                                         const float* __restrict__ packed,
                                                         const int32_t* __restrict__ pos,
                                                         const int32_t* __restrict__ cnt, int n_layers,
                                                         const int64_t* __restrict__ layer_off,
                                                         float* __restrict__ dst,
                                                         const float* __restrict__ Zi, float* __restrict__ Vd,
                                                         const float* __restrict__ z_prev /* RES only */,
                                                         double* __restrict__ part /* RES only */)
{
    static_assert(DUAL || !RES, "the residual sums are formed with the dual update");
    double s_ro = 0.0, s_so = 0.0;
    // stores 4 (or 1) elements of z at arena element e and, with DUAL, updates Vd there
    auto put4 = [&](int64_t e, const v4f& z) {
        st4(dst + e, z);
        if (DUAL) {
            const v4f zi = ld4(Zi + e);
            const v4f d = zi - z;
            st4(Vd + e, ld4(Vd + e) + d);
            if (RES) {
                s_ro = sqd4(s_ro, zi, z);
                s_so = sqd4(s_so, z, ld4(z_prev + e));
            }
        }
    };
    auto put1 = [&](int64_t e, float z) {
        dst[e] = z;
        if (DUAL) {
            const float zi = Zi[e];
            const float d = zi - z;
            Vd[e] = Vd[e] + d;
            if (RES) {
                s_ro = sqd(s_ro, zi, z);
                s_so = sqd(s_so, z, z_prev[e]);
            }
        }
    };
    const WorkItem it = items[blockIdx.x];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int row_len = it.row_len;
    const float* in = packed + layer_off[it.layer];
    const v4f zero4 = {0.f, 0.f, 0.f, 0.f};
    if (!mode_has_channels(item_mode(it))) {
        const int lpr = it.lpr <= kWave ? it.lpr : kBlock;
        const int rows_at_once = kBlock / lpr;
        const int sub = threadIdx.x / lpr;
        const int j = threadIdx.x - sub * lpr;
        for (int rr = sub; rr < it.nr; rr += rows_at_once) {
            const int p = pos[it.g0 + rr];
            const int64_t d = it.base + (int64_t)rr * row_len;
            const float* s = in + (int64_t)(p < 0 ? 0 : p) * row_len;
            if (item_vec(it)) {
                const int nchunk = row_len >> 2;
                if (p >= 0) for (int c = j; c < nchunk; c += lpr) put4(d + 4 * c, ld4u(s + 4 * c));
                else for (int c = j; c < nchunk; c += lpr) put4(d + 4 * c, zero4);
            } else {
                if (p >= 0) for (int c = j; c < row_len; c += lpr) put1(d + c, s[c]);
                else for (int c = j; c < row_len; c += lpr) put1(d + c, 0.f);
            }
        }
    } else {
        // a wave takes a row of dst; a lane fills 4 adjacent columns (kept ones from the packed row,
        // the others +0) and stores them with one 128-bit access.  BOTH: the row of a pruned filter
        // is all +0, the row of a kept one is read at its rank among the kept filters.
        const bool both = item_mode(it) == HSADMM_MODE_BOTH;
        const int kc = both ? cnt[2 * n_layers + it.layer] : cnt[it.layer];
        const int khw = it.khw;
        const int in_len = kc * khw;
        const DivKhw div(khw);
        const int32_t* pl = pos + (both ? it.aux : (int64_t)it.g0);
        const int quads = item_vec(it) ? (row_len >> 2) : 0;
        // Two 128-bit stores in flight per lane: of two rows of the wave, or, when only one row is left for it, of two
        // column groups of that row.
        constexpr int kSlots = 2;
        const WaveShare ws(it.nr, wave);
        auto cols = [&](int c) -> int4 {          // packed column of each of the dst columns c .. c + 3, -1: pruned channel
            int4 p;
            if (khw == 1) {
                __builtin_memcpy(&p, pl + c, 16);
            } else {
                const int h0 = div(c), h1 = div(c + 1), h2 = div(c + 2), h3 = div(c + 3);
                const int p0 = pl[h0], p1 = pl[h1], p2 = pl[h2], p3 = pl[h3];
                p.x = p0 >= 0 ? p0 * khw + (c - h0 * khw) : -1;
                p.y = p1 >= 0 ? p1 * khw + (c + 1 - h1 * khw) : -1;
                p.z = p2 >= 0 ? p2 * khw + (c + 2 - h2 * khw) : -1;
                p.w = p3 >= 0 ? p3 * khw + (c + 3 - h3 * khw) : -1;
            }
            return p;
        };
        for (int rr0 = ws.row; rr0 < it.nr; rr0 += kSlots * ws.rows_at_once) {
            const bool one_row = rr0 + ws.rows_at_once >= it.nr;
            int prow[kSlots], coff[kSlots];
            const float* srow[kSlots];
            int64_t drow[kSlots];
#pragma unroll
            for (int u = 0; u < kSlots; ++u) {
                const int rr = one_row ? rr0 : rr0 + u * ws.rows_at_once;
                prow[u] = both ? pos[it.g0 + rr] : it.row0 + rr;
                srow[u] = in + (int64_t)(prow[u] < 0 ? 0 : prow[u]) * in_len;
                drow[u] = it.base + (int64_t)rr * row_len;
                coff[u] = one_row ? u * ws.stride : 0;
            }
            const int step = one_row ? kSlots * ws.stride : ws.stride;
            for (int c4 = lane + ws.first; c4 < quads; c4 += step) {
                int4 p[kSlots];
                bool on[kSlots];
                v4f v[kSlots];
#pragma unroll
                for (int u = 0; u < kSlots; ++u) {
                    on[u] = c4 + coff[u] < quads;
                    p[u] = (on[u] && prow[u] >= 0) ? cols((c4 + coff[u]) << 2) : int4{-1, -1, -1, -1};
                }
#pragma unroll
                for (int u = 0; u < kSlots; ++u) {
                    v[u].x = p[u].x >= 0 ? srow[u][p[u].x] : 0.f;
                    v[u].y = p[u].y >= 0 ? srow[u][p[u].y] : 0.f;
                    v[u].z = p[u].z >= 0 ? srow[u][p[u].z] : 0.f;
                    v[u].w = p[u].w >= 0 ? srow[u][p[u].w] : 0.f;
                }
#pragma unroll
                for (int u = 0; u < kSlots; ++u)
                    if (on[u]) put4(drow[u] + ((int64_t)(c4 + coff[u]) << 2), v[u]);
            }
            for (int c = (quads << 2) + lane + ws.first; c < row_len; c += ws.stride) {
                const int ch = div(c);
                const int p0 = pl[ch];
                const int pc = p0 >= 0 ? p0 * khw + (c - ch * khw) : -1;
#pragma unroll
                for (int u = 0; u < (one_row ? 1 : kSlots); ++u)
                    put1(drow[u] + c, (prow[u] >= 0 && pc >= 0) ? srow[u][pc] : 0.f);
            }
        }
    }
    if (RES) block_sum_pair(s_ro, s_so, part + (int64_t)blockIdx.x * 4 + 2);
}

}  // namespace
#endif
