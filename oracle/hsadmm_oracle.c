/*
 * CPU oracle for the per-layer structured-sparsity step of H-SADMM.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the plain definition of what the
 * step computes, written as scalar loops so it can be checked against the
 * paper by eye.  It shares no code, header, table or constant with the HIP
 * library and must never be called from the product path: only the tests, the
 * smoke check and the benchmark's cpu_baseline leg load it.
 *
 * Build:  gcc -O2 -ffp-contract=off -fopenmp -shared -fPIC  (no -ffast-math)
 *
 * Layer l is the row-major fp32 array W[c_out][c_in][khw] (Section 2, first
 * paragraph; linear layers have khw = 1) stored at elem_off[l] in every
 * full-layout arena.  Groups (Section 2.1, "Structured Sparsity Constraints"):
 *     mode 1, filter  g:  W[g, :, :]   (G = c_out)
 *     mode 2, channel g:  W[:, g, :]   (G = c_in)
 *     mode 0, none:       unconstrained layer (Section 2.1, last sentence);
 *                         its c_out filters are all kept.
 *     mode 4, shape   g:  W[:, b, u, v] with g = b*khw + (u,v)   (G = c_in*khw): shape
 *                         sparsity of Section 2.1, one group per spatial position of an input
 *                         channel, i.e. per column of the [c_out][c_in*khw] GEMM view
 *     mode 3, both:       the intersection S_f ^ S_c of Section 2.1: c_out filter
 *                         groups followed by c_in channel groups (G = c_out + c_in);
 *                         k filters and k_in channels are kept.
 *     mode 5, channel ^ shape:  S_c ^ S_s of Section 2.1: c_in channel groups followed by c_in*khw
 *                         shape groups (G = c_in + c_in*khw); k_in channels and k_kern shape groups
 *                         are kept.
 *     mode 6, all three:  S_f ^ S_c ^ S_s, the composite set of Section 2.1 in full: c_out filter
 *                         groups, c_in channel groups, c_in*khw shape groups (G = their sum);
 *                         k filters, k_in channels, k_kern shape groups are kept.
 *                         Modes 5 and 6 are defined for the projection (oracle_project,
 *                         oracle_project_weighted) only: the other functions take such a layer
 *                         through its GEMM view, where the shape groups are the columns (mode 2,
 *                         or mode 3 with the filters), and refuse these two modes.
 * Mask and key arrays hold the groups of all layers, concatenated in table
 * order.
 *
 * OpenMP only distributes independent elements / groups / rows over threads;
 * the order of floating-point operations inside every element and every group
 * is the same for any thread count, so results are bit-identical to a
 * single-threaded run.
 *
 * Parity pins: tests/test_oracle_*.py (hand-worked layers, brute-force
 * projection optimality, rank-count vs stable sort, library-routine special
 * cases, invariants).  No function here is "parity unpinned".
 */
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#include <math.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORACLE_NONE = 0, ORACLE_FILTER = 1, ORACLE_CHANNEL = 2, ORACLE_BOTH = 3, ORACLE_SHAPE = 4,
       ORACLE_CHANNEL_SHAPE = 5, ORACLE_ALL = 6 };

static int g_threads = 1;

void oracle_set_threads(int t)
{
    g_threads = t < 1 ? 1 : t;
#ifdef _OPENMP
    omp_set_num_threads(g_threads);
#endif
}

int oracle_get_threads(void) { return g_threads; }

/* Groups of a layer in mask / key (see the list of modes above). */
static int64_t n_groups(int mode, int c_out, int c_in, int khw)
{
    if (mode == ORACLE_SHAPE) return (int64_t)c_in * khw;
    if (mode == ORACLE_BOTH) return (int64_t)c_out + c_in;
    if (mode == ORACLE_CHANNEL_SHAPE) return (int64_t)c_in + (int64_t)c_in * khw;
    if (mode == ORACLE_ALL) return (int64_t)c_out + c_in + (int64_t)c_in * khw;
    return mode == ORACLE_CHANNEL ? c_in : c_out;
}

/* The counts of a layer are in range for its mode (k_kern may be NULL when the mode does not read it). */
static int counts_ok(int mode, int64_t co, int64_t ci, int64_t s, int64_t k, int64_t k_in, const int32_t *k_kern,
                     int32_t l)
{
    if (mode == ORACLE_NONE) return 1;
    if (mode == ORACLE_BOTH) return k >= 1 && k <= co && k_in >= 1 && k_in <= ci;
    if (mode == ORACLE_CHANNEL_SHAPE || mode == ORACLE_ALL) {
        if (!k_kern) return 0;
        if (mode == ORACLE_ALL && (k < 1 || k > co)) return 0;
        return k_in >= 1 && k_in <= ci && k_kern[l] >= 1 && k_kern[l] <= k_in * s;
    }
    if (mode < ORACLE_NONE || mode > ORACLE_ALL) return 0;
    return k >= 1 && k <= n_groups(mode, (int)co, (int)ci, (int)s);
}

/*
 * One projection onto "at most kk nonzero groups" (Eq. (10) and the paragraph after it), applied in
 * place to the layer x[co][ci][s]: squared Frobenius norm of every group of x as it stands
 * (sequential fp64 sum in memory order), rank count (larger key first, lower index first among
 * equals), +0 written over the groups not kept.  channel = 0: groups are filters x[g,:,:];
 * channel = 1: groups are input channels x[:,g,:]; channel = 2: groups are the shape positions
 * x[:,b,t] with g = b*s + t.  key, m: the G entries of this constraint.
 */
static void project_in_place(float *x, int64_t co, int64_t ci, int64_t s, int channel, int64_t kk,
                             double *key, uint8_t *m)
{
    const int64_t G = channel == 2 ? ci * s : (channel ? ci : co);
#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < G; ++g) {
        double acc = 0.0;
        if (channel == 2) {
            for (int64_t o = 0; o < co; ++o) {
                const double y = (double)x[o * ci * s + g];
                acc += y * y;
            }
        } else if (channel) {
            for (int64_t o = 0; o < co; ++o)
                for (int64_t t = 0; t < s; ++t) {
                    const double y = (double)x[(o * ci + g) * s + t];
                    acc += y * y;
                }
        } else {
            for (int64_t t = 0; t < ci * s; ++t) {
                const double y = (double)x[g * ci * s + t];
                acc += y * y;
            }
        }
        key[g] = acc;
    }
#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < G; ++g) {
        int64_t before = 0;
        for (int64_t h = 0; h < G; ++h)
            if (key[h] > key[g] || (key[h] == key[g] && h < g)) ++before;
        m[g] = before < kk ? 1 : 0;
    }
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < co * ci * s; ++e) {
        const int64_t g = channel == 2 ? e % (ci * s) : (channel ? (e / s) % ci : e / (ci * s));
        if (!m[g]) x[e] = 0.0f;
    }
}

/*
 * Composite projection for S = S_f ^ S_c (Section 2.1; Section 3, paragraph after Eq. (10)): the
 * individual projections applied one after the other, the filter projection first, the channel
 * projection on its output.  The channel norms are therefore those of the tensor whose pruned
 * filters are already zero.  (The channels selected can differ from those the opposite order
 * selects: the paper's remark that the order does not matter holds for which kind of group each
 * projection removes, rows or columns of the GEMM view, not for the selection itself.)
 * key, m: c_out filter entries followed by c_in channel entries.
 */
static void project_composite(float *x, int64_t co, int64_t ci, int64_t s, int64_t k_out, int64_t k_in,
                              double *key, uint8_t *m)
{
    project_in_place(x, co, ci, s, 0, k_out, key, m);
    project_in_place(x, co, ci, s, 1, k_in, key + co, m + co);
}

/*
 * The shape projection when a channel projection has gone before it (S_c ^ S_s, Section 2.1; the
 * projections one after the other, Section 3, paragraph after Eq. (10)): the positions of a pruned
 * channel are zero already and are not candidates; of the positions of the kept channels (cm[b] != 0),
 * the kk of largest norm are kept (equal norms: lower index first).  The norms are those of x as it
 * stands; key and m get all ci*s entries (m = 0 for a position of a pruned channel).
 * Applying the plain shape projection to x instead would give the same x: a position of a pruned
 * channel has norm 0, so where the plain ranking prefers it to a candidate, that candidate is zero
 * too.  Only the mask can differ then (it would name positions of pruned channels); this form keeps
 * the mask inside the support of the channel projection.
 */
static void project_shapes_within(float *x, int64_t co, int64_t ci, int64_t s, int64_t kk, const uint8_t *cm,
                                  double *key, uint8_t *m)
{
    const int64_t G = ci * s;
#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < G; ++g) {
        double acc = 0.0;
        for (int64_t o = 0; o < co; ++o) {
            const double y = (double)x[o * G + g];
            acc += y * y;
        }
        key[g] = acc;
    }
#pragma omp parallel for schedule(static)
    for (int64_t g = 0; g < G; ++g) {
        int64_t before = 0;
        if (!cm[g / s]) { m[g] = 0; continue; }
        for (int64_t h = 0; h < G; ++h)
            if (cm[h / s] && (key[h] > key[g] || (key[h] == key[g] && h < g))) ++before;
        m[g] = before < kk ? 1 : 0;
    }
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < co * G; ++e)
        if (!m[e % G]) x[e] = 0.0f;
}

/*
 * Composite projection for S_c ^ S_s (filters = 0) and S_f ^ S_c ^ S_s (filters = 1), Section 2.1:
 * the individual projections one after the other in the order the paper lists the sets, filters,
 * then channels, then shape groups, each on the output of the one before.
 * key, m: (c_out filter entries,) c_in channel entries, c_in*s shape entries.
 */
static void project_nested(float *x, int64_t co, int64_t ci, int64_t s, int filters, int64_t k_out, int64_t k_in,
                           int64_t k_kern, double *key, uint8_t *m)
{
    if (filters) {
        project_in_place(x, co, ci, s, 0, k_out, key, m);
        key += co;
        m += co;
    }
    project_in_place(x, co, ci, s, 1, k_in, key, m);
    project_shapes_within(x, co, ci, s, k_kern, m, key + ci, m + ci);
}

/*
 * Steps (a)-(d) for every layer.  (A layer under both constraints takes (b) and (c) from
 * project_composite above; k_in is read for such layers only.  k_kern is read for layers of modes 5
 * and 6 only and may be NULL when the table has none.)
 *
 *  (a) consensus average: Eq. (9) with lambda = 0 and rho_2 = 0 is the plain
 *      mean over the node's replicas; summed left to right in fp32, then
 *      multiplied by fl32(1/R).
 *  (b) candidate V = Wbar + U (the buffer of Algorithm 1, Phase 2) and the
 *      squared Frobenius norm of each group (Section 2.1), accumulated
 *      sequentially in fp64 in increasing memory order.  No square root is
 *      taken: the ranking is the same and no two distinct keys can merge.
 *  (c) Euclidean projection onto "at most k nonzero groups" (Eq. (10) and the
 *      paragraph after it): keep the k groups of largest norm; equal norms
 *      are ranked by lower group index.  Z = V on kept groups, +0 elsewhere.
 *  (d) dual update U <- U + (Wbar - Z), parenthesised as in Eq. (12).
 *
 * W: array of R pointers to full-layout arenas.  U: in/out.  Z, mask, key:
 * out.  Wbar: out, may be NULL.  Returns 0, or -1 on a bad argument, -2 on a
 * non-finite input.
 */
int oracle_project(int32_t L, const int64_t *elem_off, const int32_t *c_out, const int32_t *c_in,
                   const int32_t *khw, const int32_t *mode, const int32_t *k, const int32_t *k_in,
                   const int32_t *k_kern, const float *const *W, int32_t R, float *U, float *Z, float *Wbar,
                   uint8_t *mask, double *key)
{
    if (L < 1 || R < 1 || !W || !U || !Z || !mask || !key || !k_in) return -1;
    const float inv_R = 1.0f / (float)R;
    int64_t gbase = 0;
    for (int32_t l = 0; l < L; ++l) {
        const int64_t co = c_out[l], ci = c_in[l], s = khw[l];
        const int64_t n = co * ci * s;
        const int64_t G = n_groups(mode[l], c_out[l], c_in[l], khw[l]);
        if (co < 1 || ci < 1 || s < 1) return -1;
        if (!counts_ok(mode[l], co, ci, s, k[l], k_in[l], k_kern, l)) return -1;
        const int64_t off = elem_off[l];
        float *wbar = (float *)malloc(sizeof(float) * (size_t)n);
        float *v = (float *)malloc(sizeof(float) * (size_t)n);
        if (!wbar || !v) { free(wbar); free(v); return -1; }
        int bad = 0;

        /* (a), (b): elementwise mean and candidate */
#pragma omp parallel for schedule(static) reduction(| : bad)
        for (int64_t e = 0; e < n; ++e) {
            float acc = W[0][off + e];
            for (int32_t r = 1; r < R; ++r) acc = acc + W[r][off + e];
            wbar[e] = acc * inv_R;
            v[e] = wbar[e] + U[off + e];
            if (!isfinite(v[e])) bad = 1;
        }
        if (bad) { free(wbar); free(v); return -2; }

        if (mode[l] >= ORACLE_BOTH) {
            /* (b), (c) under several constraints, or under shape sparsity: v becomes Pi_S(v); then (d) */
            if (mode[l] == ORACLE_BOTH) project_composite(v, co, ci, s, k[l], k_in[l], key + gbase, mask + gbase);
            else if (mode[l] == ORACLE_SHAPE) project_in_place(v, co, ci, s, 2, k[l], key + gbase, mask + gbase);
            else project_nested(v, co, ci, s, mode[l] == ORACLE_ALL, k[l], k_in[l], k_kern[l], key + gbase, mask + gbase);
#pragma omp parallel for schedule(static)
            for (int64_t e = 0; e < n; ++e) {
                Z[off + e] = v[e];
                U[off + e] = U[off + e] + (wbar[e] - v[e]);
                if (Wbar) Wbar[off + e] = wbar[e];
            }
            free(wbar);
            free(v);
            gbase += G;
            continue;
        }

        /* (b): one fp64 key per group */
        double *kl = key + gbase;
        if (mode[l] == ORACLE_CHANNEL) {
#pragma omp parallel for schedule(static)
            for (int64_t g = 0; g < G; ++g) {
                double acc = 0.0;
                for (int64_t o = 0; o < co; ++o)
                    for (int64_t t = 0; t < s; ++t) {
                        const double x = (double)v[(o * ci + g) * s + t];
                        acc += x * x;
                    }
                kl[g] = acc;
            }
        } else {
            const int64_t gs = ci * s;
#pragma omp parallel for schedule(static)
            for (int64_t g = 0; g < G; ++g) {
                double acc = 0.0;
                for (int64_t t = 0; t < gs; ++t) {
                    const double x = (double)v[g * gs + t];
                    acc += x * x;
                }
                kl[g] = acc;
            }
        }

        /* (c): rank count. Group g is kept iff fewer than k groups precede it
         * in the order "larger key first, lower index first among equals". */
        uint8_t *ml = mask + gbase;
        if (mode[l] == ORACLE_NONE) {
            for (int64_t g = 0; g < G; ++g) ml[g] = 1;
        } else {
            const int64_t kk = k[l];
#pragma omp parallel for schedule(static)
            for (int64_t g = 0; g < G; ++g) {
                int64_t before = 0;
                for (int64_t h = 0; h < G; ++h)
                    if (kl[h] > kl[g] || (kl[h] == kl[g] && h < g)) ++before;
                ml[g] = before < kk ? 1 : 0;
            }
        }

        /* (c) projection and (d) dual update */
#pragma omp parallel for schedule(static)
        for (int64_t e = 0; e < n; ++e) {
            int64_t g;
            if (mode[l] == ORACLE_CHANNEL) g = (e / s) % ci;
            else g = e / (ci * s);
            const float z = ml[g] ? v[e] : 0.0f;
            Z[off + e] = z;
            U[off + e] = U[off + e] + (wbar[e] - z);
            if (Wbar) Wbar[off + e] = wbar[e];
        }
        free(wbar);
        free(v);
        gbase += G;
    }
    return 0;
}

/* Index sets of Section 4.4.1 ("Tensor Shrinkage"): the kept filters and kept channels of layer l,
 * ascending (the order nonzero-extraction gives).  A filter mask keeps all
 * channels, a channel mask keeps all filters, mode none keeps both whole; with
 * both constraints the filter bytes ml[0..co) and the channel bytes
 * ml[co..co+ci) each give their own set. */
static void index_sets(int mode, int64_t co, int64_t ci, const uint8_t *ml,
                       int32_t *k_out, int64_t *n_out, int32_t *k_in, int64_t *n_in)
{
    int64_t a = 0, b = 0;
    const uint8_t *mc = mode == ORACLE_BOTH ? ml + co : ml;      /* channel bytes */
    for (int64_t o = 0; o < co; ++o)
        if ((mode != ORACLE_FILTER && mode != ORACLE_BOTH) || ml[o]) k_out[a++] = (int32_t)o;
    for (int64_t c = 0; c < ci; ++c)
        if ((mode != ORACLE_CHANNEL && mode != ORACLE_BOTH) || mc[c]) k_in[b++] = (int32_t)c;
    *n_out = a;
    *n_in = b;
}

/*
 * Step (e1), tensor shrinkage (Section 4.4.1, Eq. (15)): for every layer
 *     packed[layer_off[l] + (p*|K_in| + q)*khw + t] = src[l][K_out[p]][K_in[q]][t]
 * with layer_off[0] = 0 and layer_off[l+1] = roundup(layer_off[l] + size_l,
 * pack_align).  Offsets are in elements.  kept_idx receives, layer after
 * layer, the ascending layer-local indices of the kept groups (for mode none:
 * 0..c_out-1; for both constraints: the kept filters, then the kept channels).  Padding elements of `packed` are not written.  The number of
 * kept groups comes from the mask, not from a k.
 * Returns 0 or -1.  *n_kept_idx (may be NULL) receives the entries written
 * to kept_idx.
 */
int oracle_compact(int32_t L, const int64_t *elem_off, const int32_t *c_out, const int32_t *c_in,
                   const int32_t *khw, const int32_t *mode, int32_t pack_align,
                   const float *src, const uint8_t *mask,
                   float *packed, int64_t *layer_off, int32_t *kept_idx, int64_t *n_kept_idx)
{
    if (L < 1 || pack_align < 1 || !src || !mask || !packed || !layer_off || !kept_idx) return -1;
    int64_t gbase = 0, pos = 0, nk = 0;
    layer_off[0] = 0;
    for (int32_t l = 0; l < L; ++l) {
        const int64_t co = c_out[l];
        int64_t ci = c_in[l], s = khw[l];
        int lm = mode[l];
        const int64_t G = n_groups(mode[l], c_out[l], c_in[l], khw[l]);
        if (mode[l] > ORACLE_SHAPE) return -1;            /* modes 5, 6: through the GEMM view only */
        if (lm == ORACLE_SHAPE) {
            /* shape groups are the columns of the [c_out][c_in*khw] view: packed like channels of width 1 */
            ci *= s;
            s = 1;
            lm = ORACLE_CHANNEL;
        }
        int32_t *k_out = (int32_t *)malloc(sizeof(int32_t) * (size_t)co);
        int32_t *k_in = (int32_t *)malloc(sizeof(int32_t) * (size_t)ci);
        if (!k_out || !k_in) { free(k_out); free(k_in); return -1; }
        int64_t n_out, n_in;
        index_sets(lm, co, ci, mask + gbase, k_out, &n_out, k_in, &n_in);
        const float *sl = src + elem_off[l];
        float *pl = packed + pos;
#pragma omp parallel for schedule(static)
        for (int64_t p = 0; p < n_out; ++p)
            for (int64_t q = 0; q < n_in; ++q)
                for (int64_t t = 0; t < s; ++t)
                    pl[(p * n_in + q) * s + t] = sl[((int64_t)k_out[p] * ci + k_in[q]) * s + t];
        if (lm != ORACLE_CHANNEL)
            for (int64_t p = 0; p < n_out; ++p) kept_idx[nk++] = k_out[p];
        if (lm == ORACLE_CHANNEL || lm == ORACLE_BOTH)
            for (int64_t q = 0; q < n_in; ++q) kept_idx[nk++] = k_in[q];
        pos += n_out * n_in * s;
        pos = (pos + pack_align - 1) / pack_align * pack_align;
        layer_off[l + 1] = pos;
        free(k_out);
        free(k_in);
        gbase += G;
    }
    if (n_kept_idx) *n_kept_idx = nk;
    return 0;
}

/*
 * Step (e2), recovery (Section 4.4.3, "Recovery and Consistency", and its unnumbered equation): dst is
 * set to +0 everywhere, then dst[l][K_out[p]][K_in[q]][t] = packed[...p,q,t].
 * Layer offsets inside `packed` are recomputed from the mask exactly as in
 * oracle_compact.
 */
int oracle_expand(int32_t L, const int64_t *elem_off, const int32_t *c_out, const int32_t *c_in,
                  const int32_t *khw, const int32_t *mode, int32_t pack_align,
                  const float *packed, const uint8_t *mask, float *dst)
{
    if (L < 1 || pack_align < 1 || !packed || !mask || !dst) return -1;
    int64_t gbase = 0, pos = 0;
    for (int32_t l = 0; l < L; ++l) {
        const int64_t co = c_out[l];
        int64_t ci = c_in[l], s = khw[l];
        int lm = mode[l];
        const int64_t G = n_groups(mode[l], c_out[l], c_in[l], khw[l]);
        if (mode[l] > ORACLE_SHAPE) return -1;            /* modes 5, 6: through the GEMM view only */
        if (lm == ORACLE_SHAPE) { ci *= s; s = 1; lm = ORACLE_CHANNEL; }     /* as in oracle_compact */
        int32_t *k_out = (int32_t *)malloc(sizeof(int32_t) * (size_t)co);
        int32_t *k_in = (int32_t *)malloc(sizeof(int32_t) * (size_t)ci);
        if (!k_out || !k_in) { free(k_out); free(k_in); return -1; }
        int64_t n_out, n_in;
        index_sets(lm, co, ci, mask + gbase, k_out, &n_out, k_in, &n_in);
        float *dl = dst + elem_off[l];
        const float *pl = packed + pos;
        const int64_t n = co * ci * s;
#pragma omp parallel for schedule(static)
        for (int64_t e = 0; e < n; ++e) dl[e] = 0.0f;
#pragma omp parallel for schedule(static)
        for (int64_t p = 0; p < n_out; ++p)
            for (int64_t q = 0; q < n_in; ++q)
                for (int64_t t = 0; t < s; ++t)
                    dl[((int64_t)k_out[p] * ci + k_in[q]) * s + t] = pl[(p * n_in + q) * s + t];
        pos += n_out * n_in * s;
        pos = (pos + pack_align - 1) / pack_align * pack_align;
        free(k_out);
        free(k_in);
        gbase += G;
    }
    return 0;
}

/*
 * Retraining branch of Algorithm 1, Phase 3 (Section 4.5, "Mask Freezing and Retraining Phase"): once the
 * masks are frozen the projection is replaced by the element-wise application of the cached mask,
 *     z = z~ (.) m,
 * with the same candidate z~ = Wbar + U (steps (a), (b)) and the same dual update (d) as oracle_project.
 * mask: in, nonzero = kept, any number of kept groups per layer (a union of node masks keeps more than k);
 * groups of an unconstrained layer are kept whatever their mask bytes say; under shape sparsity an entry
 * takes the byte of its (channel, position) column; under both constraints an
 * entry is kept iff its filter byte and its channel byte are both nonzero.  Entries of a masked-out
 * group are exactly +0 (as the projection writes them), whatever the sign of the candidate.
 * Returns 0, -1 on a bad argument, -2 on a non-finite candidate.
 */
int oracle_project_frozen(int32_t L, const int64_t *elem_off, const int32_t *c_out, const int32_t *c_in,
                          const int32_t *khw, const int32_t *mode,
                          const float *const *W, int32_t R, float *U, float *Z, float *Wbar,
                          const uint8_t *mask)
{
    if (L < 1 || R < 1 || !W || !U || !Z || !mask) return -1;
    const float inv_R = 1.0f / (float)R;
    int64_t gbase = 0;
    for (int32_t l = 0; l < L; ++l) {
        const int64_t co = c_out[l], ci = c_in[l], s = khw[l];
        if (co < 1 || ci < 1 || s < 1) return -1;
        const int64_t n = co * ci * s;
        const int64_t G = n_groups(mode[l], c_out[l], c_in[l], khw[l]);
        if (mode[l] > ORACLE_SHAPE) return -1;            /* modes 5, 6: through the GEMM view only */
        const int64_t off = elem_off[l];
        const uint8_t *ml = mask + gbase;
        int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
        for (int64_t e = 0; e < n; ++e) {
            float acc = W[0][off + e];
            for (int32_t r = 1; r < R; ++r) acc = acc + W[r][off + e];
            const float wbar = acc * inv_R;
            const float v = wbar + U[off + e];
            if (!isfinite(v)) bad = 1;
            int64_t g;
            if (mode[l] == ORACLE_SHAPE) g = e % (ci * s);
            else if (mode[l] == ORACLE_CHANNEL) g = (e / s) % ci;
            else g = e / (ci * s);
            int keep = mode[l] == ORACLE_NONE || ml[g] != 0;          /* both: g is the filter */
            if (mode[l] == ORACLE_BOTH) keep = keep && ml[co + (e / s) % ci] != 0;
            const float z = keep ? v : 0.0f;
            Z[off + e] = z;
            U[off + e] = U[off + e] + (wbar - z);
            if (Wbar) Wbar[off + e] = wbar;
        }
        if (bad) return -2;
        gbase += G;
    }
    return 0;
}

/*
 * Bitwise mask synchronisation (Section 4.3, Eq. (14)): out = OR over the M masks, byte by byte
 * (any nonzero byte counts as "kept"; the result holds 0 / 1).
 */
int oracle_mask_or(int64_t n_groups_total, const uint8_t *const *masks, int32_t M, uint8_t *out)
{
    if (n_groups_total < 0 || M < 1 || !masks || !out) return -1;
    for (int64_t g = 0; g < n_groups_total; ++g) {
        uint8_t any = 0;
        for (int32_t i = 0; i < M; ++i) any |= masks[i][g] != 0 ? 1 : 0;
        out[g] = any;
    }
    return 0;
}

/*
 * Mask drift (Section 4.5, "Mask Freezing and Retraining Phase": the masks are frozen once the sparsity pattern has
 * stopped changing): per layer, the number of groups whose kept flag differs between two masks (any nonzero byte
 * counts as kept).  An unconstrained layer keeps all its groups whatever its bytes say, so its drift is 0.
 */
int oracle_mask_drift(int32_t L, const int32_t *c_out, const int32_t *c_in, const int32_t *khw, const int32_t *mode,
                      const uint8_t *a, const uint8_t *b, int32_t *drift)
{
    if (L < 1 || !a || !b || !drift) return -1;
    int64_t gbase = 0;
    for (int32_t l = 0; l < L; ++l) {
        const int64_t G = n_groups(mode[l], c_out[l], c_in[l], khw[l]);
        if (mode[l] > ORACLE_SHAPE) return -1;            /* modes 5, 6: through the GEMM view only */
        int32_t d = 0;
        if (mode[l] != ORACLE_NONE)
            for (int64_t g = 0; g < G; ++g) d += ((a[gbase + g] != 0) != (b[gbase + g] != 0)) ? 1 : 0;
        drift[l] = d;
        gbase += G;
    }
    return 0;
}

/*
 * Weights of the dense node candidate, Eq. (9): with P accelerators per node, M nodes, weight decay
 * lambda and the layer's penalties rho_1, rho_2,
 *     gamma = lambda / M + P rho_1 + rho_2,
 *     z~ = (1/gamma) [ rho_1 sum_j (theta_j + u_j) + rho_2 (z - v) ] = a (Wbar + U) + b (z - v)
 * where Wbar and U are the means over the node's P replicas, a = P rho_1 / gamma, b = rho_2 / gamma.
 * Computed in fp64, rounded once to fp32.  Returns 0, or -1 on a bad argument (gamma <= 0 included).
 */
int oracle_node_coefficients(int32_t L, const double *rho1, const double *rho2, double lambda, int32_t M,
                             int32_t P, float *a, float *b)
{
    if (L < 1 || !rho1 || !rho2 || !a || !b || M < 1 || P < 1) return -1;
    for (int32_t l = 0; l < L; ++l) {
        const double gamma = lambda / (double)M + (double)P * rho1[l] + rho2[l];
        if (!(gamma > 0.0) || rho1[l] < 0.0 || rho2[l] < 0.0) return -1;
        a[l] = (float)((double)P * rho1[l] / gamma);
        b[l] = (float)(rho2[l] / gamma);
    }
    return 0;
}

/*
 * Steps (a)-(d) with the full candidate of Eq. (9):
 *     Wbar as in oracle_project;  t = Wbar + U;  q = Zg - Vd  (global consensus minus inter-node dual);
 *     z~ = fl(fl(a_l t) + fl(b_l q))   in fp32, no fused multiply-add;
 *     keys, selection and Z = Pi_S(z~) as in oracle_project (Eq. (10));
 *     U <- U + (Wbar - Z)  (Eq. (12): the intra-node dual update involves theta and z_i only).
 * Zg, Vd: in, full-layout arenas.  a, b: L fp32 weights.  Other arguments as for oracle_project.
 */
int oracle_project_weighted(int32_t L, const int64_t *elem_off, const int32_t *c_out, const int32_t *c_in,
                            const int32_t *khw, const int32_t *mode, const int32_t *k, const int32_t *k_in,
                            const int32_t *k_kern, const float *const *W, int32_t R, float *U, const float *Zg, const float *Vd,
                            const float *a, const float *b, float *Z, float *Wbar, uint8_t *mask, double *key)
{
    if (L < 1 || R < 1 || !W || !U || !Zg || !Vd || !a || !b || !Z || !mask || !key || !k_in) return -1;
    const float inv_R = 1.0f / (float)R;
    int64_t gbase = 0;
    for (int32_t l = 0; l < L; ++l) {
        const int64_t co = c_out[l], ci = c_in[l], s = khw[l];
        if (co < 1 || ci < 1 || s < 1) return -1;
        const int64_t n = co * ci * s;
        const int64_t G = n_groups(mode[l], c_out[l], c_in[l], khw[l]);
        if (!counts_ok(mode[l], co, ci, s, k[l], k_in[l], k_kern, l)) return -1;
        const int64_t off = elem_off[l];
        float *wbar = (float *)malloc(sizeof(float) * (size_t)n);
        float *v = (float *)malloc(sizeof(float) * (size_t)n);
        if (!wbar || !v) { free(wbar); free(v); return -1; }
        int bad = 0;
        const float al = a[l], bl = b[l];
#pragma omp parallel for schedule(static) reduction(| : bad)
        for (int64_t e = 0; e < n; ++e) {
            float acc = W[0][off + e];
            for (int32_t r = 1; r < R; ++r) acc = acc + W[r][off + e];
            wbar[e] = acc * inv_R;
            const float t = wbar[e] + U[off + e];
            const float q = Zg[off + e] - Vd[off + e];
            const float at = al * t;
            const float bq = bl * q;
            v[e] = at + bq;
            if (!isfinite(v[e])) bad = 1;
        }
        if (bad) { free(wbar); free(v); return -2; }
        if (mode[l] >= ORACLE_BOTH) {
            if (mode[l] == ORACLE_BOTH) project_composite(v, co, ci, s, k[l], k_in[l], key + gbase, mask + gbase);
            else if (mode[l] == ORACLE_SHAPE) project_in_place(v, co, ci, s, 2, k[l], key + gbase, mask + gbase);
            else project_nested(v, co, ci, s, mode[l] == ORACLE_ALL, k[l], k_in[l], k_kern[l], key + gbase, mask + gbase);
#pragma omp parallel for schedule(static)
            for (int64_t e = 0; e < n; ++e) {
                Z[off + e] = v[e];
                U[off + e] = U[off + e] + (wbar[e] - v[e]);
                if (Wbar) Wbar[off + e] = wbar[e];
            }
            free(wbar);
            free(v);
            gbase += G;
            continue;
        }
        double *kl = key + gbase;
#pragma omp parallel for schedule(static)
        for (int64_t g = 0; g < G; ++g) {
            double acc = 0.0;
            if (mode[l] == ORACLE_CHANNEL) {
                for (int64_t o = 0; o < co; ++o)
                    for (int64_t t = 0; t < s; ++t) {
                        const double x = (double)v[(o * ci + g) * s + t];
                        acc += x * x;
                    }
            } else {
                for (int64_t t = 0; t < ci * s; ++t) {
                    const double x = (double)v[g * ci * s + t];
                    acc += x * x;
                }
            }
            kl[g] = acc;
        }
        uint8_t *ml = mask + gbase;
        if (mode[l] == ORACLE_NONE) {
            for (int64_t g = 0; g < G; ++g) ml[g] = 1;
        } else {
            const int64_t kk = k[l];
#pragma omp parallel for schedule(static)
            for (int64_t g = 0; g < G; ++g) {
                int64_t before = 0;
                for (int64_t h = 0; h < G; ++h)
                    if (kl[h] > kl[g] || (kl[h] == kl[g] && h < g)) ++before;
                ml[g] = before < kk ? 1 : 0;
            }
        }
#pragma omp parallel for schedule(static)
        for (int64_t e = 0; e < n; ++e) {
            int64_t g;
            if (mode[l] == ORACLE_CHANNEL) g = (e / s) % ci;
            else g = e / (ci * s);
            const float z = ml[g] ? v[e] : 0.0f;
            Z[off + e] = z;
            U[off + e] = U[off + e] + (wbar[e] - z);
            if (Wbar) Wbar[off + e] = wbar[e];
        }
        free(wbar);
        free(v);
        gbase += G;
    }
    return 0;
}

/*
 * The retraining branch of Algorithm 1, Phase 3, with the full candidate: z_i = z~ (.) m for a given (frozen) mask m,
 * where z~ is the dense node candidate of Eq. (9) exactly as oracle_project_weighted forms it
 * (z~ = fl(fl(a_l t) + fl(b_l q)), t = Wbar + U, q = Zg - Vd), followed by the dual update of Eq. (12),
 * U <- U + (Wbar - Z).  No norms and no selection.  The mask is read as in oracle_project_frozen (any nonzero byte
 * = kept; the groups of an unconstrained layer are kept whatever their bytes say; an element of a layer under both
 * constraints is kept iff its filter byte and its channel byte are nonzero).
 */
int oracle_project_weighted_frozen(int32_t L, const int64_t *elem_off, const int32_t *c_out, const int32_t *c_in,
                                   const int32_t *khw, const int32_t *mode, const float *const *W, int32_t R,
                                   float *U, const float *Zg, const float *Vd, const float *a, const float *b,
                                   float *Z, float *Wbar, const uint8_t *mask)
{
    if (L < 1 || R < 1 || !W || !U || !Zg || !Vd || !a || !b || !Z || !mask) return -1;
    const float inv_R = 1.0f / (float)R;
    int64_t gbase = 0;
    for (int32_t l = 0; l < L; ++l) {
        const int64_t co = c_out[l], ci = c_in[l], s = khw[l];
        if (co < 1 || ci < 1 || s < 1) return -1;
        const int64_t n = co * ci * s;
        const int64_t G = n_groups(mode[l], c_out[l], c_in[l], khw[l]);
        if (mode[l] > ORACLE_SHAPE) return -1;            /* modes 5, 6: through the GEMM view only */
        const int64_t off = elem_off[l];
        const uint8_t *ml = mask + gbase;
        const float al = a[l], bl = b[l];
        int bad = 0;
#pragma omp parallel for schedule(static) reduction(| : bad)
        for (int64_t e = 0; e < n; ++e) {
            float acc = W[0][off + e];
            for (int32_t r = 1; r < R; ++r) acc = acc + W[r][off + e];
            const float wbar = acc * inv_R;
            const float t = wbar + U[off + e];
            const float q = Zg[off + e] - Vd[off + e];
            const float at = al * t;
            const float bq = bl * q;
            const float zt = at + bq;
            if (!isfinite(zt)) bad = 1;
            int64_t g;
            if (mode[l] == ORACLE_SHAPE) g = e % (ci * s);
            else if (mode[l] == ORACLE_CHANNEL) g = (e / s) % ci;
            else g = e / (ci * s);
            int keep = mode[l] == ORACLE_NONE || ml[g] != 0;          /* both: g is the filter */
            if (mode[l] == ORACLE_BOTH) keep = keep && ml[co + (e / s) % ci] != 0;
            const float z = keep ? zt : 0.0f;
            Z[off + e] = z;
            U[off + e] = U[off + e] + (wbar - z);
            if (Wbar) Wbar[off + e] = wbar;
        }
        if (bad) return -2;
        gbase += G;
    }
    return 0;
}

/*
 * Global consensus, Eq. (11): z = (1/M) sum_i (z_i + v_i).  The terms c_i = z_i + v_i arrive as M buffers of
 * equal length (the compacted pre-transmission buffers of Section 4.4.2, all under the same mask); the sum runs
 * left to right in fp32 in node order and is multiplied by fl32(1/M), the convention of the replica mean.
 */
int oracle_average(int32_t M, int64_t n, const float *const *bufs, float *out)
{
    if (M < 1 || n < 0 || !bufs || !out) return -1;
    const float inv_M = 1.0f / (float)M;
#pragma omp parallel for schedule(static)
    for (int64_t e = 0; e < n; ++e) {
        float acc = bufs[0][e];
        for (int32_t i = 1; i < M; ++i) acc = acc + bufs[i][e];
        out[e] = acc * inv_M;
    }
    return 0;
}

/*
 * Inter-node dual update, Eq. (13): v <- v + (z_i - z), element by element over every layer (arena
 * padding is left alone).  Zi: the node's projected consensus; Zg: the new global consensus.
 */
int oracle_dual_inter(int32_t L, const int64_t *elem_off, const int32_t *c_out, const int32_t *c_in,
                      const int32_t *khw, const float *Zi, const float *Zg, float *Vd)
{
    if (L < 1 || !Zi || !Zg || !Vd) return -1;
    for (int32_t l = 0; l < L; ++l) {
        const int64_t n = (int64_t)c_out[l] * c_in[l] * khw[l];
        const int64_t off = elem_off[l];
#pragma omp parallel for schedule(static)
        for (int64_t e = 0; e < n; ++e) Vd[off + e] = Vd[off + e] + (Zi[off + e] - Zg[off + e]);
    }
    return 0;
}

/*
 * Pre-transmission buffer of Section 4.4.1: c = z_i + v_i (fp32), element by element over every layer,
 * into a full-layout arena that oracle_compact then shrinks (Algorithm 1, Phase 4).
 */
int oracle_add_arenas(int32_t L, const int64_t *elem_off, const int32_t *c_out, const int32_t *c_in,
                      const int32_t *khw, const float *A, const float *B, float *C)
{
    if (L < 1 || !A || !B || !C) return -1;
    for (int32_t l = 0; l < L; ++l) {
        const int64_t n = (int64_t)c_out[l] * c_in[l] * khw[l];
        const int64_t off = elem_off[l];
#pragma omp parallel for schedule(static)
        for (int64_t e = 0; e < n; ++e) C[off + e] = A[off + e] + B[off + e];
    }
    return 0;
}

/*
 * Layer-wise squared residual norms of Section 3.4 (last paragraph) / Algorithm 1 Phase 5, in fp64,
 * accumulated sequentially in memory order (differences are formed in fp64 from the fp32 values):
 *     out[0*L + l] = sum_j || theta_j - z_i ||_F^2      intra-node primal, summed over the node's R replicas
 *     out[1*L + l] = || z_i - z_i_prev ||_F^2           intra-node dual, without its rho_1 factor
 *     out[2*L + l] = || z_i - z ||_F^2                  inter-node primal
 *     out[3*L + l] = || z - z_prev ||_F^2               inter-node dual, without its rho_2 factor
 * Zi_prev, Zg, Zg_prev may be NULL; rows whose operands are missing are set to 0.
 */
int oracle_residuals(int32_t L, const int64_t *elem_off, const int32_t *c_out, const int32_t *c_in,
                     const int32_t *khw, const float *const *W, int32_t R, const float *Zi,
                     const float *Zi_prev, const float *Zg, const float *Zg_prev, double *out)
{
    if (L < 1 || R < 1 || !W || !Zi || !out) return -1;
    for (int32_t l = 0; l < L; ++l) {
        const int64_t n = (int64_t)c_out[l] * c_in[l] * khw[l];
        const int64_t off = elem_off[l];
        double r_in = 0.0, s_in = 0.0, r_out = 0.0, s_out = 0.0;
        for (int64_t e = 0; e < n; ++e) {
            const double zi = (double)Zi[off + e];
            for (int32_t r = 0; r < R; ++r) {
                const double d = (double)W[r][off + e] - zi;
                r_in += d * d;
            }
            if (Zi_prev) { const double d = zi - (double)Zi_prev[off + e]; s_in += d * d; }
            if (Zg) { const double d = zi - (double)Zg[off + e]; r_out += d * d; }
            if (Zg && Zg_prev) { const double d = (double)Zg[off + e] - (double)Zg_prev[off + e]; s_out += d * d; }
        }
        out[0 * (int64_t)L + l] = r_in;
        out[1 * (int64_t)L + l] = s_in;
        out[2 * (int64_t)L + l] = r_out;
        out[3 * (int64_t)L + l] = s_out;
    }
    return 0;
}

/*
 * Adaptive penalty tuning (Section 3.4, last paragraph; Algorithm 1, Phase 5, last line).  The paper adopts, per
 * layer and independently for rho_1 and rho_2, the residual-balancing rule of the ADMM reference it cites (Boyd et
 * al., Section 3.4.1 there): with the norms ||r|| and ||s|| of the primal and dual residuals,
 *     rho <- tau_incr * rho   if ||r|| > mu ||s||
 *     rho <- rho / tau_decr   if ||s|| > mu ||r||
 *     rho unchanged           otherwise,
 * and, the duals being scaled ones (u = y / rho), a dual is multiplied by rho_old / rho_new when its rho changes.
 * mu, tau_incr, tau_decr are not given in the paper: arguments.  The caps rho_1^max, rho_2^max are those of the
 * paper's hyperparameter paragraph (Section 5): a raised penalty stops at its cap.
 * Norms, from the squared sums sq[4L] laid out as oracle_residuals writes them and the residuals of Section 3.4:
 *   intra:  ||r||^2 = sq[0L + l]  (r_intra,i,j summed over the node's P replicas);
 *           ||s||^2 = P rho_1^2 sq[1L + l]  (s_intra,i,j = rho_1 (z_i^{k+1} - z_i^k), the same for each of the P)
 *   inter:  ||r||^2 = sq[2L + l];  ||s||^2 = n_out rho_2^2 sq[3L + l], n_out = the number of nodes whose r_inter
 *           were added into sq[2L + l] (1: the node's own view)
 * rho1, rho2: in/out, L doubles;  scale_u, scale_v: out, L floats, rho_old / rho_new rounded once.
 */
int oracle_adapt_penalties(int32_t L, const double *sq, int32_t P, int32_t n_out, double mu, double tau_incr,
                           double tau_decr, double rho1_max, double rho2_max, double *rho1, double *rho2,
                           float *scale_u, float *scale_v)
{
    if (L < 1 || !sq || !rho1 || !rho2 || !scale_u || !scale_v || P < 1 || n_out < 1) return -1;
    if (!(mu > 0.0) || !(tau_incr >= 1.0) || !(tau_decr >= 1.0)) return -1;
    for (int32_t l = 0; l < L; ++l) {
        if (!(rho1[l] > 0.0) || !(rho2[l] > 0.0) || rho1[l] > rho1_max || rho2[l] > rho2_max) return -1;
        for (int k = 0; k < 4; ++k)
            if (!(sq[(int64_t)k * L + l] >= 0.0)) return -1;
    }
    for (int32_t l = 0; l < L; ++l) {
        for (int level = 0; level < 2; ++level) {
            double *rho = level == 0 ? &rho1[l] : &rho2[l];
            const double cap = level == 0 ? rho1_max : rho2_max;
            const double copies = level == 0 ? (double)P : (double)n_out;
            const double r = sqrt(sq[(int64_t)(2 * level) * L + l]);
            const double s = *rho * sqrt(copies * sq[(int64_t)(2 * level + 1) * L + l]);
            const double old = *rho;
            double next = old;
            if (r > mu * s) {
                next = tau_incr * old;
                if (next > cap) next = cap;
            } else if (s > mu * r) {
                next = old / tau_decr;
            }
            *rho = next;
            (level == 0 ? scale_u : scale_v)[l] = (float)(old / next);
        }
    }
    return 0;
}

/* X[e] <- fl(X[e] * factor[l]) on every element of every layer (the rescaling of a scaled dual after its layer's
 * penalty has changed; arena padding untouched). */
int oracle_scale_layers(int32_t L, const int64_t *elem_off, const int32_t *c_out, const int32_t *c_in,
                        const int32_t *khw, const float *factor, float *X)
{
    if (L < 1 || !factor || !X) return -1;
    for (int32_t l = 0; l < L; ++l) {
        const int64_t n = (int64_t)c_out[l] * c_in[l] * khw[l];
        const int64_t off = elem_off[l];
        const float f = factor[l];
#pragma omp parallel for num_threads(g_threads) schedule(static)
        for (int64_t e = 0; e < n; ++e) X[off + e] = X[off + e] * f;
    }
    return 0;
}

/*
 * Layer-wise squared Frobenius norms of one arena, in fp64, accumulated sequentially in memory order:
 *     out[l] = sum over layer l of (double)X[e]^2
 * (the magnitudes the feasibility thresholds of Section 3.4 are relative to).
 */
int oracle_layer_sqnorms(int32_t L, const int64_t *elem_off, const int32_t *c_out, const int32_t *c_in,
                         const int32_t *khw, const float *X, double *out)
{
    if (L < 1 || !X || !out) return -1;
    for (int32_t l = 0; l < L; ++l) {
        const int64_t n = (int64_t)c_out[l] * c_in[l] * khw[l];
        const int64_t off = elem_off[l];
        double s = 0.0;
        for (int64_t e = 0; e < n; ++e) {
            const double x = (double)X[off + e];
            s += x * x;
        }
        out[l] = s;
    }
    return 0;
}

/*
 * Stopping test (Section 3.4, last paragraph; Algorithm 1, Phase 5: "if R_pri < eps_pri and R_dual < eps_dual then
 * break").  The paper declares a layer converged once its total primal and dual residual norms fall below
 * feasibility thresholds built from an absolute and a relative tolerance as in the ADMM reference it cites (Boyd
 * et al., Section 3.3.1 there):
 *     eps_pri  = sqrt(p) eps_abs + eps_rel max(||A x||, ||B z||),      eps_dual = sqrt(p) eps_abs + eps_rel ||A^T y||.
 * Written out for the two consensus levels of this method, for one layer of n elements, P replicas per node and the
 * contributions of n_out nodes added up (1: a node's own view).  The constraints are theta_ij - z_i = 0 (P per node)
 * and z_i - z = 0 (one per node), p = (P + 1) n n_out scalars in all; "A x" stacks theta_i1..theta_iP and z_i, "B z"
 * stacks P copies of z_i and one of z, and y stacks the unscaled duals rho_1 u_ij and rho_2 v_i:
 *     R_pri^2  = sq[0L + l] + sq[2L + l]                          (all primal residuals of Section 3.4)
 *     R_dual^2 = P rho_1^2 sq[1L + l] + n_out rho_2^2 sq[3L + l]  (all dual residuals; s_intra is the same for each replica)
 *     ||A x||^2   = mag[0L + l] + mag[1L + l]                     (sum_j ||theta_j||^2 ; ||z_i||^2)
 *     ||B z||^2   = P mag[1L + l] + n_out mag[2L + l]             (||z||^2)
 *     ||A^T y||^2 = rho_1^2 mag[3L + l] + rho_2^2 mag[4L + l]     (sum_j ||u_j||^2 ; ||v_i||^2)
 * sq: 4L squared residual sums as oracle_residuals writes them; mag: 5L squared magnitudes (sum_j ||theta_j||^2,
 * ||z_i||^2, ||z||^2, sum_j ||u_j||^2, ||v_i||^2; with several nodes each summed over them, ||z||^2 excepted).
 * done[l] = 1 iff R_pri < eps_pri and R_dual < eps_dual (strictly, as Algorithm 1 prints it); *all_done = 1 iff every
 * layer is done.  eps_abs, eps_rel >= 0 are arguments: the paper gives neither.
 */
int oracle_stopping_test(int32_t L, const int64_t *n_elems, int32_t P, int32_t n_out, const double *rho1,
                         const double *rho2, const double *sq, const double *mag, double eps_abs, double eps_rel,
                         int32_t *done, int32_t *all_done)
{
    if (L < 1 || !n_elems || !rho1 || !rho2 || !sq || !mag || !done || !all_done || P < 1 || n_out < 1) return -1;
    if (!(eps_abs >= 0.0) || !(eps_rel >= 0.0)) return -1;
    for (int32_t l = 0; l < L; ++l) {
        if (n_elems[l] < 1 || !(rho1[l] > 0.0) || !(rho2[l] > 0.0)) return -1;
        for (int k = 0; k < 4; ++k) if (!(sq[(int64_t)k * L + l] >= 0.0)) return -1;
        for (int k = 0; k < 5; ++k) if (!(mag[(int64_t)k * L + l] >= 0.0)) return -1;
    }
    int32_t every = 1;
    for (int32_t l = 0; l < L; ++l) {
        const double r_pri = sqrt(sq[0 * (int64_t)L + l] + sq[2 * (int64_t)L + l]);
        const double r_dual = sqrt((double)P * rho1[l] * rho1[l] * sq[1 * (int64_t)L + l] +
                                   (double)n_out * rho2[l] * rho2[l] * sq[3 * (int64_t)L + l]);
        const double p = (double)(P + 1) * (double)n_elems[l] * (double)n_out;
        const double ax = sqrt(mag[0 * (int64_t)L + l] + mag[1 * (int64_t)L + l]);
        const double bz = sqrt((double)P * mag[1 * (int64_t)L + l] + (double)n_out * mag[2 * (int64_t)L + l]);
        const double aty = sqrt(rho1[l] * rho1[l] * mag[3 * (int64_t)L + l] + rho2[l] * rho2[l] * mag[4 * (int64_t)L + l]);
        const double eps_pri = sqrt(p) * eps_abs + eps_rel * (ax > bz ? ax : bz);
        const double eps_dual = sqrt(p) * eps_abs + eps_rel * aty;
        done[l] = (r_pri < eps_pri && r_dual < eps_dual) ? 1 : 0;
        if (!done[l]) every = 0;
    }
    *all_done = every;
    return 0;
}
