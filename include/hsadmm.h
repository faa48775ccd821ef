/*
 * hsadmm.h -- C ABI of the MI355X (gfx950) library for the per-layer
 * structured-sparsity step of H-SADMM (PruneX, arXiv 2512.14628).
 *
 * The step is what a node runs between local training and inter-node
 * synchronisation (Algorithm 1, Phases 2-5, restricted to one device):
 *
 *   (a) consensus average of R replica weight buffers     Eq. (9) with lambda = 0, rho_2 = 0
 *   (b) candidate V = Wbar + U and per-group squared norm  Algorithm 1 Phase 2; Section 2.1
 *   (c) per-layer top-k group selection, Z = Pi_S(V)       Eq. (10) and the paragraph after it
 *   (d) dual update U <- U + (Wbar - Z)                    Eq. (12)
 *   (e) tensor shrinkage / recovery of the kept groups     Section 4.4.1 Eq. (15); Section 4.4.3
 *
 * and, around it: the frozen-mask branch and the mask union (Section 4.5, Eq. (14)), the full node
 * candidate with its rho_2 term, the inter-node dual update and the mean of the nodes' compact
 * buffers (Eq. (9), (13), (11)), the residual norms and the adaptive penalties they drive (Section 3.4)
 * and the mask drift (Section 4.5).
 * Each projection (hsadmm_project, _frozen, _weighted, _weighted_frozen) also exists as a *_compact call that returns the
 * shrunk buffer as well, with the same results as the projection followed by the compaction.
 * hsadmm_step is the one entry point behind all of these forms (an argument structure; the named calls are it with
 * fields left NULL).  It also takes the previous outer iteration's selection as a prediction (Section 4.5: the
 * pattern stops changing after a few iterations), which changes no result and makes a step whose selection comes
 * out as predicted touch every element once; and it forms the intra-node residual norms on the way.
 * hsadmm_stopping_test (host) is the break test of Algorithm 1's Phase 5.
 *
 * Data layout.  A layer is the row-major fp32 array W[c_out][c_in][khw]
 * (Section 2, first paragraph; khw = K_H*K_W, 1 for linear layers).  A
 * "full-layout arena" is one device buffer that holds every layer at the
 * element offset `elem_off` of its table entry; all arenas passed to one plan
 * (each replica, U, Z, Wbar, src, dst) share that table.  Groups (Section
 * 2.1): FILTER group g = W[g,:,:] (G = c_out), CHANNEL group g = W[:,g,:]
 * (G = c_in); a NONE layer is unconstrained and contributes G = c_out groups
 * that are always kept.  A BOTH layer carries the intersection S_f ^ S_c of
 * Section 2.1: its c_out filter groups are followed by its c_in channel
 * groups (G = c_out + c_in), k filters and k_in channels are kept, and an
 * element survives iff its filter and its channel both do.  `mask` and
 * `sqnorm` hold the groups of all layers concatenated in table order.
 * Shape sparsity (groups W[:, b, u, v], one per input channel and spatial
 * position) needs no mode of its own: such a group is a column of the
 * [c_out][c_in*khw] view, so declare the layer as CHANNEL with c_in*khw
 * channels and khw = 1 (BOTH, the same way, for filters together with shapes).
 * Shape groups together with channel groups (S_c ^ S_s, S_f ^ S_c ^ S_s) are such a
 * layer plus a limit on the runs of K_H*K_W columns that may hold kept columns:
 * hsadmm_plan_create_nested.
 *
 * Ownership.  The caller owns every device buffer and the stream.  The
 * library owns only the plan (host tables plus a device copy, allocated in
 * hsadmm_plan_create on the current device and released in
 * hsadmm_plan_destroy).  Apart from plan creation / destruction and
 * hsadmm_plan_set_node_weights (a synchronous copy into the plan; the `coef`
 * field of hsadmm_step avoids it), no call allocates or frees memory or
 * synchronises the device; each enqueues all its work on `hip_stream`
 * (a hipStream_t passed as void*; NULL is the default stream), so a sequence
 * of calls can be captured into a HIP graph.  Outputs are
 * valid once the caller has synchronised that stream.  The workspace also
 * carries the index mappings of the compaction (kept positions, counts,
 * offsets) from the call that derives them to the calls that reuse them, so
 * calls that share a workspace must be ordered on one stream.
 *
 * Device.  A plan belongs to the HIP device that was current in
 * hsadmm_plan_create; every later call on it must be made with that device
 * current (INVALID_ARGUMENT otherwise) and with buffers of that device.
 *
 * Errors.  Every call returns HSADMM_OK (0) or a negative code.  Arguments
 * are validated before anything is enqueued, so a call that returns an
 * argument error has had no effect on device memory.  No exceptions cross
 * the boundary.  Calls on one plan from several host threads are safe when
 * each uses its own workspace (with the per-kernel timing diagnostics on, see
 * hsadmm_kernel_timing_enable for what is and is not).
 *
 * Preconditions that are not checked: all input values are finite; buffers
 * do not alias except where stated.
 */
#ifndef HSADMM_H
#define HSADMM_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define HSADMM_OK                     0
#define HSADMM_ERR_INVALID_ARGUMENT  -1   /* null pointer, bad size, bad table entry, misaligned pointer */
#define HSADMM_ERR_WORKSPACE         -2   /* workspace_bytes smaller than hsadmm_plan_sizes reports */
#define HSADMM_ERR_HIP               -3   /* a HIP runtime call or a kernel launch failed */
#define HSADMM_ERR_UNSUPPORTED       -4   /* valid request beyond a compiled limit (R > HSADMM_MAX_REPLICAS, ...) */
#define HSADMM_ERR_HOST_MEMORY       -5   /* a host allocation failed while a plan's tables were built */

#define HSADMM_MODE_NONE     0
#define HSADMM_MODE_FILTER   1
#define HSADMM_MODE_CHANNEL  2
#define HSADMM_MODE_BOTH     3   /* FILTER | CHANNEL: both constraints on one layer */

#define HSADMM_MAX_REPLICAS  16
#define HSADMM_MAX_LAYERS    4096
#define HSADMM_MAX_MASKS     64

/* One table entry per layer.  Host memory, caller-owned, copied by hsadmm_plan_create. */
typedef struct {
    int64_t elem_off;   /* offset of the layer, in elements, in every full-layout arena; multiple of 4 */
    int32_t c_out;      /* >= 1 */
    int32_t c_in;       /* >= 1 */
    int32_t khw;        /* >= 1; K_H*K_W, 1 for linear layers */
    int32_t mode;       /* HSADMM_MODE_* */
    int32_t k;          /* groups kept (the paper's alpha), 1 <= k <= G; ignored for MODE_NONE;
                           MODE_BOTH: filters kept (alpha_out), 1 <= k <= c_out */
    int32_t k_in;       /* MODE_BOTH only: channels kept (alpha_in), 1 <= k_in <= c_in; ignored otherwise */
} hsadmm_layer_t;

typedef struct hsadmm_plan hsadmm_plan_t;   /* opaque; its tables never change after creation */

/*
 * Build a plan for a table of L layers (1 <= L <= HSADMM_MAX_LAYERS).
 * Layers must not overlap and must appear in increasing elem_off order.
 * pack_align_elems >= 1: every layer's segment of the packed buffer starts
 * at a multiple of this many elements (1 = tight packing).
 * Needs a HIP device (tables are copied to the current device).
 * Errors: INVALID_ARGUMENT (table), UNSUPPORTED (more than 2^31 - 1 groups in all),
 * HOST_MEMORY (host allocation failure), HIP (no device / device allocation failure).
 */
int hsadmm_plan_create(const hsadmm_layer_t* layers, int32_t L, int32_t pack_align_elems,
                       hsadmm_plan_t** out);

/*
 * Shape groups inside input channels (Section 2.1: the composite set's S_c ^ S_s and
 * S_f ^ S_c ^ S_s; the projections one after the other, Section 3, paragraph after
 * Eq. (10), in the order the sets are listed: filters, channels, shape groups).
 *
 * A shape group W[:, b, u, v] is a column of the layer's [c_out][c_in*K_H*K_W] GEMM view, so a
 * layer under shape sparsity is declared through that view: c_in = C_in*K_H*K_W channels with
 * khw = 1, MODE_CHANNEL (or MODE_BOTH with the filters), k (k_in) = shape groups kept.  The
 * columns of one input channel are then a run of `span` = K_H*K_W consecutive channels of the
 * view.  An entry with span >= 1 limits the runs as well: the selection first ranks the runs by
 * the sum of their channels' squared norms (the input channel's norm; MODE_BOTH: over the kept
 * filters) and keeps k_coarse of them, lower index first among equals, then ranks the channels
 * of the kept runs alone and keeps k (k_in) of them.  Channels of a pruned run are never
 * candidates, so exactly k (k_in) channels are kept and all of them lie in kept runs; the
 * values equal those of the plain shape projection applied after the channel projection.
 * mask, sqnorm, sel and the index mappings keep the layout of the layer as declared (one entry
 * per channel of the view; the runs have no entries of their own: a run is kept iff one of its
 * channels is); sqnorm reports 0 for a channel of a pruned run, its norm once the run is zero.
 * Every call that takes the plan works as for any CHANNEL / BOTH layer.
 *
 * nest: NULL (then this is hsadmm_plan_create), or L entries, host memory, copied.  An entry
 * with span <= 0 sets no limit (k_coarse is ignored).  An entry with span >= 1 needs
 * MODE_CHANNEL or MODE_BOTH, khw == 1, c_in a multiple of span, 1 <= k_coarse <= c_in / span
 * and k (MODE_BOTH: k_in) <= k_coarse * span, else INVALID_ARGUMENT.  Other arguments and
 * errors as for hsadmm_plan_create.
 */
typedef struct {
    int32_t span;       /* channels of the view per run (K_H*K_W; 1 for a 1x1 layer); <= 0: no limit on runs */
    int32_t k_coarse;   /* runs that may hold kept channels (the paper's alpha_in) */
} hsadmm_nest_t;

int hsadmm_plan_create_nested(const hsadmm_layer_t* layers, const hsadmm_nest_t* nest, int32_t L,
                              int32_t pack_align_elems, hsadmm_plan_t** out);

/* Releases the plan's host and device memory.  NULL is ignored.  The caller
 * must have synchronised every stream that still runs work of this plan. */
void hsadmm_plan_destroy(hsadmm_plan_t* plan);

/*
 * Sizes a caller needs to allocate buffers (any output pointer may be NULL):
 *   arena_elems            minimum length of a full-layout arena, in elements
 *   groups_total           length of mask / sqnorm / kept_idx
 *   packed_capacity_elems  length of `packed` that fits any mask
 *   workspace_bytes        size of the scratch buffer the calls with a workspace argument take
 */
int hsadmm_plan_sizes(const hsadmm_plan_t* plan, int64_t* arena_elems, int64_t* groups_total,
                      int64_t* packed_capacity_elems, size_t* workspace_bytes);

/*
 * Steps (a)-(d) for every layer of the plan.
 *
 *   W_replicas  HOST array of R DEVICE pointers, each a full-layout arena (read only)
 *   R           1 <= R <= HSADMM_MAX_REPLICAS
 *   U           device, in/out: the (replica-mean) scaled dual variable, updated in place
 *   Z           device, out: the projected node consensus; +0 on pruned groups
 *   Wbar        device, out, may be NULL: the consensus average
 *   mask        device, out, groups_total bytes: 1 = group kept; exactly k ones per constrained layer
 *   sqnorm      device, out, may be NULL, groups_total doubles: squared Frobenius norm of each group of V
 *   workspace   device scratch of workspace_bytes >= hsadmm_plan_sizes' figure, 256-byte aligned
 *
 * Arithmetic (fp32 unless stated; no fused multiply-add across these steps):
 *   Wbar = ((W_0 + W_1) + ... + W_{R-1}) * fl32(1/R);  V = Wbar + U;
 *   sqnorm_g = sum over the group of (double)V^2, in fp64 (summation order is
 *   fixed per layer shape, the same for every group of a layer);
 *   a group is kept iff fewer than k groups of its layer have a larger
 *   sqnorm, or an equal sqnorm and a lower index;
 *   Z = V on kept groups, +0 elsewhere;  U <- U + (Wbar - Z).
 * MODE_BOTH layers (Section 3, paragraph after Eq. (10): the individual
 * projections applied one after the other): the k filters are selected from
 * the filter norms of V; the channel norms are then taken over the kept
 * filters only (the pruned ones are already zero) and the k_in channels
 * selected from them; sqnorm holds the filter norms, then these channel norms.
 *
 * All arena pointers must be 16-byte aligned.  Z, Wbar, mask, sqnorm and the
 * workspace must not alias each other or any input.  Padding elements of the
 * arenas (outside every layer) are neither read nor written.
 * Errors: INVALID_ARGUMENT, WORKSPACE, UNSUPPORTED, HIP.
 */
int hsadmm_project(const hsadmm_plan_t* plan, const float* const* W_replicas, int32_t R,
                   float* U, float* Z, float* Wbar, uint8_t* mask, double* sqnorm,
                   void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Retraining branch of Algorithm 1, Phase 3 (Section 4.5, mask freezing): the
 * projection is replaced by the element-wise application of a cached mask,
 *     Z = (Wbar + U) (.) mask,   U <- U + (Wbar - Z),
 * with the candidate formed exactly as in hsadmm_project.  One pass: every
 * replica and U are read once, Z and U written once; no norms, no selection.
 *
 *   mask   device, in, groups_total bytes, nonzero = kept; any number of kept
 *          groups per layer (e.g. the union hsadmm_mask_or gives); the groups
 *          of a MODE_NONE layer are kept whatever their bytes say; an element
 *          of a MODE_BOTH layer is kept iff its filter byte and its channel
 *          byte are both nonzero.
 * Masked-out entries of Z are exactly +0.  Other arguments, alignment and
 * aliasing rules as for hsadmm_project; no workspace is needed.
 * Errors: INVALID_ARGUMENT, UNSUPPORTED, HIP.
 */
int hsadmm_project_frozen(const hsadmm_plan_t* plan, const float* const* W_replicas, int32_t R,
                          float* U, float* Z, float* Wbar, const uint8_t* mask, void* hip_stream);

/*
 * The projection under a frozen mask and the tensor shrinkage of its result
 * in one call (Section 4.5; Section 4.4.1, Eq. (15)): the same outputs, bit
 * for bit, as hsadmm_project_frozen(...) followed by hsadmm_compact(plan, Z,
 * mask, packed, layer_off, kept_idx, ...).  Everything the mask keeps is
 * written to the packed buffer by the pass that forms it (whole rows of
 * FILTER and MODE_NONE layers, the kept channels' columns of CHANNEL and BOTH
 * layers); Z is not read again.
 *   mappings_cached  0: the index mappings are derived from the mask first
 *                    (as hsadmm_compact does when given a mask);
 *                    nonzero: the workspace already holds the index mappings
 *                    of THIS mask (left there by an earlier hsadmm_compact,
 *                    hsadmm_expand or hsadmm_project_frozen_compact that was
 *                    given it) and they are reused, as a frozen mask's cached
 *                    index sets are from iteration to iteration (Section 4.5).
 *                    The caller guarantees that such a call has run on this
 *                    plan, workspace and stream; with the mappings of another
 *                    mask of this plan the packed buffer is unspecified (no
 *                    access leaves it).
 * Other arguments, alignment, ownership and errors as for
 * hsadmm_project_frozen and hsadmm_compact.
 */
int hsadmm_project_frozen_compact(const hsadmm_plan_t* plan, const float* const* W_replicas, int32_t R,
                                  float* U, float* Z, float* Wbar, const uint8_t* mask, int32_t mappings_cached,
                                  float* packed, int64_t* layer_off, int32_t* kept_idx,
                                  void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Bitwise mask synchronisation on one device (Section 4.3, Eq. (14)):
 * out[g] = 1 if any of the M masks has a nonzero byte at g, else 0.
 *   masks  HOST array of M DEVICE pointers (1 <= M <= HSADMM_MAX_MASKS), each groups_total bytes
 *   out    device, groups_total bytes; may be one of the inputs
 * Errors: INVALID_ARGUMENT, UNSUPPORTED, HIP.
 */
int hsadmm_mask_or(const hsadmm_plan_t* plan, const uint8_t* const* masks, int32_t M, uint8_t* out,
                   void* hip_stream);

/*
 * Mask drift (Section 4.5: the masks are frozen once the sparsity pattern has
 * stopped changing): drift[l] = number of groups of layer l whose kept flag
 * (byte != 0) differs between the two masks; 0 for a MODE_NONE layer.
 *   mask_a, mask_b  device, groups_total bytes each
 *   drift           device, out, L int32
 * Errors: INVALID_ARGUMENT, HIP.
 */
int hsadmm_mask_drift(const hsadmm_plan_t* plan, const uint8_t* mask_a, const uint8_t* mask_b, int32_t* drift,
                      void* hip_stream);

/*
 * Step (e1), tensor shrinkage: packs the kept slices of `src` into one
 * contiguous dense buffer, layer after layer,
 *     packed[layer_off[l] + (p*|K_in| + q)*khw + t] = src[l][K_out[p]][K_in[q]][t]
 * where K_out / K_in are the ascending kept filter / channel indices the mask
 * gives (FILTER: K_in is every channel; CHANNEL: K_out is every filter; NONE:
 * both are everything; BOTH: each set from its own part of the mask).  The number of kept groups is read from the mask (any
 * count 0..G), not from the plan's k, so a union of several masks is valid.
 *
 *   src        device, full-layout arena (read only), 16-byte aligned
 *   mask       device, groups_total bytes, nonzero = kept; or NULL: pack under
 *              the index mappings already held in this workspace -- those of
 *              the selection the most recent hsadmm_project /
 *              hsadmm_project_weighted made (its mask, without scanning it
 *              again), or of the most recent hsadmm_compact / hsadmm_expand
 *              that was given a mask, whichever used the workspace last.
 *              With NULL the caller guarantees that one of them has run on
 *              this plan, workspace and stream.
 *   packed     device, out, at least packed_capacity_elems elements; only
 *              layer_off[L] elements are meaningful; alignment padding between
 *              segments is not written
 *   layer_off  device, out, L+1 int64: start of every layer's segment in
 *              elements; layer_off[0] = 0, layer_off[l+1] =
 *              roundup(layer_off[l] + size_l, pack_align_elems)
 *   kept_idx   device, out, groups_total int32 capacity: per layer, the
 *              ascending layer-local indices of its kept groups (BOTH: the kept
 *              filters, then the kept channels), concatenated without gaps
 *              (entries past the total kept count are not written)
 * Errors: INVALID_ARGUMENT, WORKSPACE, HIP.
 */
int hsadmm_compact(const hsadmm_plan_t* plan, const float* src, const uint8_t* mask,
                   float* packed, int64_t* layer_off, int32_t* kept_idx,
                   void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The projection step and the tensor shrinkage of its result in one call
 * (Eq. (10), Eq. (12); Section 4.4.1, Eq. (15)): the same outputs, bit for
 * bit, as hsadmm_project(...) followed by hsadmm_compact(plan, Z, NULL, packed,
 * layer_off, kept_idx, ...), i.e. Z compacted under the selection just made.
 * The compaction reads kept groups only and the repair of the speculative
 * outputs rewrites pruned groups only, so the two share one kernel launch;
 * CHANNEL layers are packed by the pass that writes their Z, and are not
 * read again.  Arguments, alignment, ownership and
 * errors as for hsadmm_project (W_replicas .. sqnorm, workspace) and
 * hsadmm_compact (packed, layer_off, kept_idx); all three compaction outputs
 * are required.  Afterwards the workspace holds the selection's index
 * mappings, as after hsadmm_project.
 */
int hsadmm_project_compact(const hsadmm_plan_t* plan, const float* const* W_replicas, int32_t R,
                           float* U, float* Z, float* Wbar, uint8_t* mask, double* sqnorm,
                           float* packed, int64_t* layer_off, int32_t* kept_idx,
                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * hsadmm_project_compact for callers that cannot allocate device memory (code
 * under HIP graph capture, tight serving loops, harnesses that forbid
 * hipMalloc) and so have no workspace to pass: the same arguments without
 * `workspace` / `workspace_bytes`, the same outputs bit for bit.  Its scratch
 * is an array of HSADMM_STATIC_SCRATCH_BYTES that the library holds statically
 * on every device it is loaded on (until the process ends); a plan whose
 * workspace_bytes (hsadmm_plan_sizes) exceed that is refused with UNSUPPORTED
 * before anything is enqueued.  The call allocates and frees nothing.
 * All calls on one device share the one array: calls that may overlap in time
 * on a device (different streams, or different plans on different streams)
 * race and must be ordered by the caller.  The array keeps the last call's
 * contents; the step writes everything it reads from it, so nothing needs
 * clearing.  The index mappings stay in that array, not in a workspace of the
 * caller's, so a later hsadmm_compact / hsadmm_expand must be given the mask.
 * Errors: UNSUPPORTED (plan too large), else those of hsadmm_project_compact.
 */
#define HSADMM_STATIC_SCRATCH_BYTES (16u << 20)
int hsadmm_project_compact_static(const hsadmm_plan_t* plan, const float* const* W_replicas, int32_t R,
                                  float* U, float* Z, float* Wbar, uint8_t* mask, double* sqnorm,
                                  float* packed, int64_t* layer_off, int32_t* kept_idx, void* hip_stream);

/*
 * Tensor shrinkage of the pre-transmission buffer c = z_i + v_i (Section
 * 4.4.1; Algorithm 1, Phase 4): exactly hsadmm_compact applied to the
 * element-wise fp32 sum src0 + src1, which is formed on the fly (no full-size
 * temporary).  src0 and src1 are full-layout arenas, 16-byte aligned.
 */
int hsadmm_compact_sum(const hsadmm_plan_t* plan, const float* src0, const float* src1, const uint8_t* mask,
                       float* packed, int64_t* layer_off, int32_t* kept_idx,
                       void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Weights of the dense node candidate, Eq. (9).  With P accelerators per
 * node, M nodes, weight decay lambda and the layer's penalties rho_1, rho_2:
 *     gamma = lambda / M + P rho_1 + rho_2
 *     z~ = (1/gamma) [ rho_1 sum_j (theta_j + u_j) + rho_2 (z - v) ]
 *        = a (Wbar + U) + b (z - v),   a = P rho_1 / gamma,  b = rho_2 / gamma
 * (Wbar, U: means over the node's P replicas).  Host function, all pointers
 * are HOST arrays of L entries; a, b are computed in fp64 and rounded once.
 * Errors: INVALID_ARGUMENT (also when some gamma <= 0 or a penalty is negative).
 */
int hsadmm_node_coefficients(const double* rho1, const double* rho2, int32_t L, double lambda, int32_t M,
                             int32_t P, float* a, float* b);

/*
 * Adaptive penalty tuning (Section 3.4, last paragraph; Algorithm 1, Phase 5,
 * last line): the residual-balancing rule of the ADMM reference the paper
 * cites (Boyd et al., "Varying penalty parameter"), applied per layer and
 * independently to rho_1 (intra-node) and rho_2 (inter-node).  With ||r|| and
 * ||s|| the norms of a level's primal and dual residuals,
 *     rho <- min(tau_incr rho, rho_max)   if ||r|| > mu ||s||
 *     rho <- rho / tau_decr               if ||s|| > mu ||r||
 *     rho unchanged                       otherwise,
 * and because u and v are scaled duals, each must be multiplied by
 * rho_old / rho_new when its penalty changes: scale_u, scale_v (feed them to
 * hsadmm_scale_layers; then recompute the node weights with
 * hsadmm_node_coefficients).  HOST function, all pointers are HOST memory.
 *   residuals  in, 4*L doubles as hsadmm_residuals / hsadmm_retrain_* write
 *              them (copied to the host by the caller).  Norms used:
 *                intra  ||r||^2 = residuals[0L+l],  ||s||^2 = P rho_1^2 residuals[1L+l]
 *                       (s_intra = rho_1 (z_i - z_i_prev) once per replica)
 *                inter  ||r||^2 = residuals[2L+l],  ||s||^2 = n_out rho_2^2 residuals[3L+l]
 *   P          replicas per node; n_out: how many nodes' inter-node primal
 *              sums were added into row 2 (1 for a node's own view)
 *   mu, tau_incr, tau_decr  the rule's constants; the paper gives none (its
 *              reference suggests 10, 2, 2).  mu > 0, tau >= 1.
 *   rho1_max, rho2_max  the caps of Section 5 (10.0 each there)
 *   rho1, rho2 in/out, L doubles, 0 < rho <= its cap
 *   scale_u, scale_v  out, L floats, rho_old / rho_new rounded once
 * Errors: INVALID_ARGUMENT (nothing is written).
 */
int hsadmm_adapt_penalties(const double* residuals, int32_t L, int32_t P, int32_t n_out,
                           double mu, double tau_incr, double tau_decr, double rho1_max, double rho2_max,
                           double* rho1, double* rho2, float* scale_u, float* scale_v);

/*
 * X <- X * factor[l] on every element of every layer l (fp32, one rounding;
 * arena padding untouched): the rescaling of a scaled dual (U or Vd) after
 * hsadmm_adapt_penalties.  Layers whose factor is exactly 1 are not touched.
 *   X       device, in/out, full-layout arena, 16-byte aligned
 *   factor  device, L floats
 * Errors: INVALID_ARGUMENT, HIP.
 */
int hsadmm_scale_layers(const hsadmm_plan_t* plan, float* X, const float* factor, void* hip_stream);

/*
 * Stores the per-layer weights a_l, b_l (HOST arrays of L floats) in the
 * plan; hsadmm_project_weighted uses them.  A new plan holds a = 1, b = 0.
 * Synchronous host-to-device copy: call it between steps (penalties adapt
 * once per outer iteration), not while a hsadmm_project_weighted of this
 * plan is in flight.  Errors: INVALID_ARGUMENT, HIP.
 */
int hsadmm_plan_set_node_weights(hsadmm_plan_t* plan, const float* a, const float* b);

/*
 * Steps (a)-(d) with the full candidate of Eq. (9):
 *     t = Wbar + U;  q = Zg - Vd;  z~ = fl(fl(a_l t) + fl(b_l q))   (fp32, no fused multiply-add)
 * then group norms, top-k and Z = Pi_S(z~) as in hsadmm_project, and the
 * intra-node dual update U <- U + (Wbar - Z) of Eq. (12).
 *   Zg   device, in: the global consensus z (full-layout arena)
 *   Vd   device, in: the node's inter-node dual v_i (full-layout arena)
 * All other arguments, alignment and aliasing rules as for hsadmm_project.
 * FILTER layers take one pass over the replicas (Z first holds Wbar + U, from
 * which either outcome of a filter is finished once the mask is known);
 * CHANNEL and BOTH layers take two passes (norms, then final values); the
 * second reads the mean of the replicas that the first parked in Z (BOTH
 * always, CHANNEL from 3 replicas on) instead of the replicas.
 * Errors: INVALID_ARGUMENT, WORKSPACE, UNSUPPORTED, HIP.
 */
int hsadmm_project_weighted(const hsadmm_plan_t* plan, const float* const* W_replicas, int32_t R,
                            float* U, const float* Zg, const float* Vd, float* Z, float* Wbar,
                            uint8_t* mask, double* sqnorm,
                            void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The weighted projection and the shrinkage of the pre-transmission buffer
 * c = z_i + v_i in one call (Eq. (9), (10), (12); Section 4.4.1; Algorithm 1,
 * Phase 4): the same outputs, bit for bit, as hsadmm_project_weighted(...)
 * followed by hsadmm_compact_sum(plan, Z, Vd, NULL, packed, layer_off,
 * kept_idx, ...).  The pass that finishes a kept filter's z~ already holds
 * its Vd, so it writes the packed row as well and the FILTER layers are not
 * read again; CHANNEL and BOTH layers are packed by their final pass, the
 * rows of unconstrained layers by workgroups of the fix-up's launch.  Arguments, alignment, ownership and errors as for
 * hsadmm_project_weighted and hsadmm_compact_sum; all three compaction
 * outputs are required.
 */
int hsadmm_project_weighted_compact(const hsadmm_plan_t* plan, const float* const* W_replicas, int32_t R,
                                    float* U, const float* Zg, const float* Vd, float* Z, float* Wbar,
                                    uint8_t* mask, double* sqnorm,
                                    float* packed, int64_t* layer_off, int32_t* kept_idx,
                                    void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * The retraining branch of Algorithm 1, Phase 3, with the full candidate of
 * Eq. (9): z_i = z~ (.) m for a given (frozen) mask m, z~ formed exactly as in
 * hsadmm_project_weighted with the plan's node weights, then the dual update
 * of Eq. (12).  No norms, no selection, one pass, no workspace.  The mask is
 * read as in hsadmm_project_frozen; Zg, Vd and the other arguments as in
 * hsadmm_project_weighted.  Errors: INVALID_ARGUMENT, UNSUPPORTED, HIP.
 */
int hsadmm_project_weighted_frozen(const hsadmm_plan_t* plan, const float* const* W_replicas, int32_t R,
                                   float* U, const float* Zg, const float* Vd, float* Z, float* Wbar,
                                   const uint8_t* mask, void* hip_stream);

/*
 * The same with the shrinkage of c = z_i + v_i under the mask in the same
 * pass (Section 4.4.1; Section 4.5): the outputs of
 * hsadmm_project_weighted_frozen(...) followed by hsadmm_compact_sum(plan, Z,
 * Vd, mask, packed, layer_off, kept_idx, ...), bit for bit.  mappings_cached,
 * workspace and the compaction outputs as in hsadmm_project_frozen_compact.
 * Together with hsadmm_expand_dual this is the whole consensus side of a
 * retraining-phase iteration in two kernel launches.
 * Errors: INVALID_ARGUMENT, WORKSPACE, UNSUPPORTED, HIP.
 */
int hsadmm_project_weighted_frozen_compact(const hsadmm_plan_t* plan, const float* const* W_replicas, int32_t R,
                                           float* U, const float* Zg, const float* Vd, float* Z, float* Wbar,
                                           const uint8_t* mask, int32_t mappings_cached,
                                           float* packed, int64_t* layer_off, int32_t* kept_idx,
                                           void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Inter-node dual update, Eq. (13): Vd <- Vd + (Zi - Zg) on every layer
 * (arena padding untouched).  Zi: the node's projected consensus; Zg: the new
 * global consensus (e.g. the output of hsadmm_expand); Vd in/out.  All three
 * are full-layout arenas, 16-byte aligned.  Errors: INVALID_ARGUMENT, HIP.
 */
int hsadmm_dual_inter(const hsadmm_plan_t* plan, const float* Zi, const float* Zg, float* Vd, void* hip_stream);

/*
 * Global consensus on one device, Eq. (11): z = (1/M) sum_i (z_i + v_i).  The
 * terms c_i = z_i + v_i are M buffers of n_elems floats each -- in the paper's
 * pipeline the nodes' compact pre-transmission buffers, which all have the
 * layout of the synchronised mask, reduced by an inter-node AllReduce and
 * divided by M (Section 4.4.2); here they are resident in one HBM:
 *     out = ((b_0 + b_1) + ... + b_{M-1}) * fl32(1/M)     (fp32, node order)
 *   bufs   HOST array of M DEVICE pointers (1 <= M <= HSADMM_MAX_MASKS), 16-byte aligned
 *   out    device, n_elems floats, 16-byte aligned; may be one of the inputs
 * The plan only carries the diagnostics; no table of it is used.
 * Errors: INVALID_ARGUMENT, UNSUPPORTED, HIP.
 */
int hsadmm_average(const hsadmm_plan_t* plan, const float* const* bufs, int32_t M, int64_t n_elems, float* out,
                   void* hip_stream);

/*
 * Layer-wise squared residual norms (Section 3.4, last paragraph; Algorithm
 * 1, Phase 5), accumulated in fp64 from the fp32 values:
 *     out[0*L + l] = sum over the R replicas of || W_r - Zi ||_F^2   (intra-node primal)
 *     out[1*L + l] = || Zi - Zi_prev ||_F^2    (intra-node dual, without its rho_1 factor)
 *     out[2*L + l] = || Zi - Zg ||_F^2         (inter-node primal)
 *     out[3*L + l] = || Zg - Zg_prev ||_F^2    (inter-node dual, without its rho_2 factor)
 * Zi_prev, Zg, Zg_prev may be NULL: rows whose operands are missing are 0.
 *   out   device, 4*L doubles.  The order of additions is fixed (results are
 *         reproducible run to run) but differs from a sequential sum.
 * hsadmm_adapt_penalties and hsadmm_stopping_test consume these norms.
 * Errors: INVALID_ARGUMENT, WORKSPACE, UNSUPPORTED, HIP.
 */
int hsadmm_residuals(const hsadmm_plan_t* plan, const float* const* W_replicas, int32_t R,
                     const float* Zi, const float* Zi_prev, const float* Zg, const float* Zg_prev,
                     double* out, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Layer-wise squared Frobenius norms of one full-layout arena, accumulated in
 * fp64 from the fp32 values: out[l] = || X_l ||_F^2 (the magnitudes the
 * thresholds of the stopping test are relative to).  The order of additions is
 * fixed, as in hsadmm_residuals.
 *   X    device, full-layout arena, 16-byte aligned;  out  device, L doubles
 * Errors: INVALID_ARGUMENT, WORKSPACE, HIP.
 */
int hsadmm_layer_sqnorms(const hsadmm_plan_t* plan, const float* X, double* out,
                         void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * Stopping test (Section 3.4, last paragraph; Algorithm 1, Phase 5: break once
 * R_pri < eps_pri and R_dual < eps_dual).  Per layer, the total primal and dual
 * residual norms over both consensus levels against the feasibility
 * thresholds of the ADMM reference the paper cites (Boyd et al., "Stopping
 * criteria"), built from an absolute and a relative tolerance.  For a layer of
 * n elements, P replicas per node and the sums of n_out nodes (1: a node's own
 * view), the constraints are theta_ij - z_i = 0 and z_i - z = 0:
 *     R_pri^2  = residuals[0L+l] + residuals[2L+l]
 *     R_dual^2 = P rho_1^2 residuals[1L+l] + n_out rho_2^2 residuals[3L+l]
 *     eps_pri  = sqrt((P+1) n n_out) eps_abs
 *                + eps_rel max( sqrt(mag[0L+l] + mag[1L+l]), sqrt(P mag[1L+l] + n_out mag[2L+l]) )
 *     eps_dual = sqrt((P+1) n n_out) eps_abs + eps_rel sqrt(rho_1^2 mag[3L+l] + rho_2^2 mag[4L+l])
 * (all in fp64; the duals enter unscaled, rho u and rho v).  HOST function,
 * all pointers are HOST memory; it needs neither a plan nor a device.
 *   n_elems     n_layers int64: elements of every layer (c_out * c_in * khw)
 *   residuals   4*L doubles as hsadmm_residuals / hsadmm_retrain_* write them
 *   magnitudes  5*L doubles, squared norms per layer (hsadmm_layer_sqnorms):
 *               sum_j ||theta_j||^2, ||z_i||^2, ||z||^2, sum_j ||u_j||^2 (P ||U||^2
 *               for a caller who holds the replica-mean dual only), ||v_i||^2
 *   rho1, rho2  L doubles, > 0;  eps_abs, eps_rel >= 0: the paper gives neither
 *   layer_done  out, L int32: 1 iff both comparisons hold strictly
 *   all_done    out: 1 iff every layer is done
 * Errors: INVALID_ARGUMENT (nothing is written).
 */
int hsadmm_stopping_test(const int64_t* n_elems, int32_t n_layers, int32_t P, int32_t n_out,
                         const double* rho1, const double* rho2, const double* residuals, const double* magnitudes,
                         double eps_abs, double eps_rel, int32_t* layer_done, int32_t* all_done);

/*
 * Step (e2), recovery: the inverse scatter.  Every element of every layer of
 * `dst` is written: kept positions receive their packed value, all others
 * exactly +0 (dst need not be cleared beforehand).  Segment offsets inside
 * `packed` are recomputed from the mask as in hsadmm_compact.
 *
 *   packed     device, read only, as produced by hsadmm_compact for this mask
 *   mask       device, groups_total bytes; or NULL: reuse the index mappings
 *              held in this workspace (the cached K_out / K_in of Section
 *              4.4.3), as described for hsadmm_compact.
 *   dst        device, out, full-layout arena, 16-byte aligned
 * Errors: INVALID_ARGUMENT, WORKSPACE, HIP.
 */
int hsadmm_expand(const hsadmm_plan_t* plan, const float* packed, const uint8_t* mask,
                  float* dst, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * hsadmm_expand with the inter-node dual update of Eq. (13) applied in the
 * same pass (Algorithm 1, Phase 4: decompress, then v_i <- v_i + z_i - z):
 * dst receives the expanded tensor, the new global consensus z, exactly as
 * hsadmm_expand writes it, and Vd <- Vd + (Zi - z) on every layer, exactly
 * as hsadmm_dual_inter computes it; z is not read back from memory.
 *   Zi   device, in: the node's projected consensus (full-layout arena)
 *   Vd   device, in/out: the node's inter-node dual (full-layout arena)
 * dst, Zi and Vd must not alias each other; 16-byte aligned.  Other arguments
 * and errors as for hsadmm_expand.
 */
int hsadmm_expand_dual(const hsadmm_plan_t* plan, const float* packed, const uint8_t* mask, float* dst,
                       const float* Zi, float* Vd, void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * A retraining-phase iteration with its convergence check (Algorithm 1,
 * Phases 3 to 5 under a frozen mask, Section 4.5; residual norms of Section
 * 3.4) in two calls that touch every tensor once: the residual norms are
 * accumulated by the kernels that form z_i and z, instead of by a pass of
 * hsadmm_residuals over W, z_i and z afterwards.
 *
 * hsadmm_retrain_project: hsadmm_project_weighted_frozen_compact (same
 * arguments, same outputs, bit for bit) except that
 *   Z          device, in/out: holds the previous z_i on entry (zeros before
 *              the first iteration), the new z_i on return
 *   residuals  device, out, 4*L doubles, 8-byte aligned, laid out as
 *              hsadmm_residuals lays out `out`: rows 0 and 1 are written,
 *                  residuals[0*L + l] = sum over the R replicas of || W_r - z_i ||_F^2
 *                  residuals[1*L + l] = || z_i - z_i(previous) ||_F^2
 *              rows 2 and 3 are left as they are.
 * hsadmm_retrain_expand: hsadmm_expand_dual (same arguments, same outputs,
 * bit for bit) and
 *   z_prev     device, in: the previous global consensus, a full-layout
 *              arena other than dst and Vd (INVALID_ARGUMENT if it overlaps
 *              either), 16-byte aligned
 *   residuals  rows 2 and 3 are written,
 *                  residuals[2*L + l] = || Zi - z ||_F^2
 *                  residuals[3*L + l] = || z - z_prev ||_F^2
 *              rows 0 and 1 are left as they are.
 * The four norms equal those of hsadmm_residuals(plan, W, R, z_i, z_i
 * (previous), z, z_prev, ...) up to the order of the fp64 additions, which is
 * fixed here too (reproducible run to run).  Each call finishes its own two
 * rows; nothing is carried from one call to the other.  hsadmm_retrain_expand
 * does not depend on the mask being frozen: after a dynamic projection
 * (hsadmm_project_weighted_compact) it gives rows 2 and 3 in the same way,
 * and hsadmm_residuals with Zg = NULL gives rows 0 and 1.
 * Errors: those of the calls they extend.
 */
int hsadmm_retrain_project(const hsadmm_plan_t* plan, const float* const* W_replicas, int32_t R,
                           float* U, const float* Zg, const float* Vd, float* Z, float* Wbar,
                           const uint8_t* mask, int32_t mappings_cached,
                           float* packed, int64_t* layer_off, int32_t* kept_idx, double* residuals,
                           void* workspace, size_t workspace_bytes, void* hip_stream);
int hsadmm_retrain_expand(const hsadmm_plan_t* plan, const float* packed, const uint8_t* mask, float* dst,
                          const float* Zi, float* Vd, const float* z_prev, double* residuals,
                          void* workspace, size_t workspace_bytes, void* hip_stream);

/*
 * One entry point for every form of the projection step (Algorithm 1, Phases
 * 2, 3 and 5 on one device): the calls above named hsadmm_project* and
 * hsadmm_retrain_project are this call with some fields left NULL, and give
 * the same results bit for bit.  Fill a zeroed hsadmm_step_args_t; a NULL
 * field means "not wanted" / "not given".
 *
 *   candidate   z~ = Wbar + U                          Zg, Vd, coef all NULL   (Eq. (9), lambda = rho_2 = 0)
 *               z~ = a_l (Wbar + U) + b_l (Zg - Vd)    Zg and Vd given         (Eq. (9))
 *   support     selected: top-k of the group norms     mask_frozen NULL        (Eq. (10))
 *               given:    z_i = z~ (.) mask_frozen     mask_frozen given       (Section 4.5, retraining branch)
 *   dual        U <- U + (Wbar - z_i) in every form                            (Eq. (12))
 *   shrinkage   of z_i (of c = z_i + Vd when Vd is given) under the support    packed, layer_off, kept_idx
 *                                                                              all three or none (Eq. (15))
 *
 * Fields (device pointers unless stated; alignment and aliasing as for the
 * named calls: arenas 16 bytes, sqnorm / layer_off / residuals 8, others 4):
 *   struct_bytes     sizeof(hsadmm_step_args_t) as the caller was compiled (INVALID_ARGUMENT if it differs)
 *   W_replicas, R    HOST array of R device arenas
 *   U                in/out; with U_out given, in only
 *   U_out            out, optional, selected support only (UNSUPPORTED with mask_frozen): the
 *                    updated dual goes here and U is left as it was (a full-layout arena that overlaps neither U
 *                    nor Z; arena padding is not written).  Under a prediction (sel_prev) the old dual then stays
 *                    readable, so rows predicted pruned are written in their final form at once (no zero fill
 *                    after the selection) and a wrong prediction is repaired from the replicas and the old dual.
 *                    CHANNEL layers and layers under both constraints then take the prediction too: written once,
 *                    in the form the record makes final, and formed again only where a layer's selection differs
 *                    from its record.
 *   Zg, Vd           in: global consensus z and the node's inter-node dual v_i
 *   coef             in, 2L floats a_0, b_0, a_1, b_1, ... (hsadmm_node_coefficients gives a and b); NULL with Zg
 *                    given: the weights stored in the plan.  Read by the kernels when they run, so a captured
 *                    graph follows the buffer's contents from replay to replay.
 *   mask_frozen      in, groups_total bytes, read as hsadmm_project_frozen reads it
 *   sel_prev         in, optional, selected support only (with Zg / Vd it needs U_out: UNSUPPORTED without;
 *                    `residuals` may be taken in the same call): the selection record of the
 *                    previous outer iteration (the `sel` output of an earlier call on this plan, or
 *                    hsadmm_selection_from_mask).  It changes no result.  It predicts which groups will be
 *                    kept (Section 4.5: the pattern stops changing after a few iterations), and FILTER layers
 *                    are then written in the form the prediction makes final and packed as they are formed:
 *                    a correct prediction leaves only a zero fill of the pruned filters' rows of Z to do after
 *                    the selection, a wrong one is repaired row by row without reading the replicas again.
 *                    A record that no call of this library wrote for this plan (ranks repeated inside a layer)
 *                    leaves Z, U, mask, sqnorm and sel correct and the packed buffer unspecified; no access
 *                    leaves the buffers.  Must not overlap `sel`.
 *   Z                out (in/out when `residuals` is given: the previous z_i on entry)
 *   Wbar, sqnorm     out, optional
 *   mask             out, required unless mask_frozen is given (then it must be NULL)
 *   sel              out, optional, groups_total int32: the selection record of this call: the rank of every
 *                    kept group among the kept groups of its layer (BOTH: of its part), -1 for a pruned group
 *   mappings_cached  as in hsadmm_project_frozen_compact (frozen support with shrinkage only)
 *   residuals        out, optional, 4L doubles: rows 0 and 1 of the residual norms of Section 3.4 (sum over the
 *                    replicas of ||W_r - z_i||^2, and ||z_i - z_i(previous)||^2), taken by the passes that form
 *                    z_i; rows 2 and 3 are left as they are (hsadmm_retrain_expand writes those).  Only with the
 *                    full candidate (Zg / Vd; UNSUPPORTED otherwise).  Given support: as hsadmm_retrain_project
 *                    (needs the shrinkage; Z brings the previous z_i).  Selected support: the previous z_i comes
 *                    in Zi_prev, and every FILTER row's sums are taken for either outcome while its replicas are
 *                    in registers and picked once the selection is known; CHANNEL and BOTH layers take theirs
 *                    from one more pass over their own replicas and final z_i.  The order of the fp64 additions
 *                    is fixed (reproducible) and differs from hsadmm_residuals'.
 *   Zi_prev          in, with `residuals` and a selected support only: the previous z_i, a full-layout arena
 *                    that overlaps neither Z nor U nor U_out
 *   workspace, workspace_bytes, hip_stream   as for the named calls (a frozen support without shrinkage needs none)
 * Errors: those of the named call that the fields select, and UNSUPPORTED for the combinations named above.
 */
typedef struct {
    size_t struct_bytes;
    const float* const* W_replicas;
    int32_t R;
    int32_t mappings_cached;
    float* U;
    float* U_out;
    const float* Zg;
    const float* Vd;
    const float* coef;
    const float* Zi_prev;
    const uint8_t* mask_frozen;
    const int32_t* sel_prev;
    float* Z;
    float* Wbar;
    uint8_t* mask;
    double* sqnorm;
    int32_t* sel;
    float* packed;
    int64_t* layer_off;
    int32_t* kept_idx;
    double* residuals;
    void* workspace;
    size_t workspace_bytes;
    void* hip_stream;
} hsadmm_step_args_t;

int hsadmm_step(const hsadmm_plan_t* plan, const hsadmm_step_args_t* args);

/*
 * The selection record of a mask (see `sel` / `sel_prev` of hsadmm_step): sel[g] = rank of group g among the
 * groups of its layer whose mask byte is nonzero (BOTH: among the filters, or among the channels), -1 where the
 * byte is zero; the groups of a MODE_NONE layer are all kept.  For a caller who holds the previous iteration's
 * mask (Algorithm 1 keeps m_i) but not its record.  Afterwards the workspace holds this mask's index mappings,
 * as after hsadmm_compact with a mask.
 * Errors: INVALID_ARGUMENT, WORKSPACE, HIP.
 */
int hsadmm_selection_from_mask(const hsadmm_plan_t* plan, const uint8_t* mask, int32_t* sel,
                               void* workspace, size_t workspace_bytes, void* hip_stream);

/* Static string for an error code (never NULL). */
const char* hsadmm_strerror(int code);

/* Library version: major*10000 + minor*100 + patch. */
int hsadmm_version(void);

/*
 * Diagnostics: per-kernel device time of the calls made on this plan.
 *
 * hsadmm_kernel_timing_enable(plan, 1) makes every kernel launch of this plan
 * carry a start/stop event pair that takes the kernel's own begin and end
 * timestamps; nothing else is put on the stream (such launches cannot be
 * captured into a graph).  At most 8192
 * launches are recorded between two reads; later launches run untimed.
 * hsadmm_kernel_timing_read waits for the recorded kernels, returns for every
 * kernel id 0..HSADMM_KERNEL_COUNT-1 the summed duration in milliseconds and
 * the number of launches, and clears the record.  This record is the only
 * part of a plan that changes after its creation: launches made from several
 * host threads claim their event pairs atomically, but enabling and reading
 * must not run while another thread is inside a call on this plan.  Off by
 * default.
 * hsadmm_kernel_grid returns the number of workgroups of the latest timed
 * launch of a kernel on this plan (0 if none was timed yet), so that a
 * profile taken elsewhere can be matched to the plan it is quoted for.
 * Errors: INVALID_ARGUMENT, HOST_MEMORY, HIP.
 */
#define HSADMM_KERNEL_COUNT 29
int hsadmm_kernel_timing_enable(hsadmm_plan_t* plan, int enable);
int hsadmm_kernel_timing_read(hsadmm_plan_t* plan, double* total_ms, int64_t* launches);
int hsadmm_kernel_grid(const hsadmm_plan_t* plan, int kernel_id);
/*
 * 1 if the un-predicted projection of this plan (hsadmm_project, hsadmm_project_compact, hsadmm_step without sel_prev,
 * dual in place) forms a prediction inside its first pass, else 0 (also for a NULL plan).  It does so for plans of
 * FILTER and unconstrained layers of 20 Mi elements or more: every FILTER layer's first rows (a sixteenth, 16 to 128)
 * are processed ahead of the rest, the key that the layer's keep ratio of them exceed estimates the layer's selection
 * threshold (Eq. (10) keeps the k largest norms), and every later row is written in the form its own key suggests --
 * kept, or pruned with the kept-form dual held in Z -- before the selection has been made.  The selection and the
 * pass after it then give every output its exact value whatever was estimated; an estimate only decides how many
 * rows that pass has to touch a second time.  Results do not depend on it; the time of a call does, a little, on how
 * the norms are ordered inside a layer.  Smaller plans and plans with CHANNEL or BOTH layers write every row in the
 * kept form and repair the pruned ones.  The published keys live in the caller's workspace, tagged with the number
 * of their call; that number comes from an atomic counter in the plan (the one thing besides the timing record that
 * a call changes in a plan; every plan counts from a start of its own), so calls from several threads stay safe and
 * plans that take turns on one workspace do not read each other's keys.  A captured graph replays its call number: a
 * replay may then use the estimate an earlier replay left, which again changes no result.  Environment, read by
 * hsadmm_plan_create: HSADMM_NO_ESTIMATE (any value)
 * switches the estimate off, HSADMM_FORCE_ESTIMATE takes it whatever the size.
 */
int hsadmm_plan_estimates(const hsadmm_plan_t* plan);
/* Name of a kernel id ("" when out of range). */
const char* hsadmm_kernel_name(int kernel_id);

#ifdef __cplusplus
}
#endif
#endif /* HSADMM_H */
