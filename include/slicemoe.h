/*
 * slicemoe.h -- C ABI of the SliceMoE layer forward pass for AMD MI355X (gfx950).
 *
 * The layer (paper Section 3, Section 3.1, Eq. 1; execution strategy of Section 3.4):
 * a token vector h in R^d is cut into S contiguous slices of width ds = d/S; a router MLP
 * shared by all slices, Linear(ds -> Hr) -> ReLU -> Linear(Hr -> E), gives logits, softmax
 * over the E experts gives p, the top-k experts of each slice are selected; expert e_j sees
 * the weighted slice p_j * x (Eq. 1) and applies a two-layer GELU MLP ds -> He -> ds; the
 * k outputs of a slice are summed and the S output slices concatenated into h' in R^d.
 * Slices bound for one expert are grouped into one stacked batch per expert (Section 3.4).
 *
 * Conventions common to every entry point
 *   - Every pointer is caller-allocated DEVICE memory unless it is the config / weights
 *     struct itself (HOST).  The library never allocates, frees or keeps a pointer.
 *   - Every call only enqueues kernels on `stream` and returns (slicemoe_backward forks one of
 *     its kernels onto a stream of the library's own and joins it back, see there); there is
 *     no host-side synchronisation and no device->host copy.  Same inputs give bit-identical
 *     outputs.
 *   - Slice id n = t*S + s; because slices are contiguous, h[T, d] row-major IS the slice
 *     matrix x[Ns = T*S, ds].  Assignment id a = n*k + j for the j-th selected expert.
 *   - Linear layers are y = x W + b with W stored [in, out] row-major; expert tensors carry
 *     the expert index on the leading axis.
 *   - dtype is the storage type of h, h' and all weights (fp32 or bf16 bit patterns);
 *     accumulation is always fp32.  topk_p is fp32, indices are int32.  The stacked expert
 *     outputs y are fp32 with fp32 storage and IEEE fp16 with bf16 storage (three more
 *     mantissa bits than bf16, so the one rounding of h' after the k-sum stays the only
 *     significant one; |y| beyond 65504 would overflow).
 *   - Limits: 1 <= k <= min(E, 8), E <= 64, d % S == 0, T*S*k < 2^31.  The matrix-core
 *     (MFMA) kernels need dtype = bf16, Hr = 256, ds in {24, 48, 64, 96, 128, 192, 384}, He % 32 == 0; any
 *     other shape runs on slower generic kernels unless SLICEMOE_FLAG_REQUIRE_MFMA is set.
 *   - Numeric range of the bf16 (matrix-core) path; nothing checks it and a value beyond it changes results without
 *     an error code.  Inputs and weights are arbitrary bf16; the limits are on intermediate values:
 *       expert layer 1   the accumulator of a hidden unit, (x W1) / 4 with the factor folded into the packed W1, is
 *                        converted to fp16 before it is scaled by p: |x W1| <= 262016 (beyond that the unit
 *                        saturates), and |p x W1 + b1| <= 262016;
 *       expert output    the stacked rows y are stored as fp16: |y| <= 65504;
 *       router layer 1   a hidden activation u = ReLU(x Wr1 + br1) enters the second layer as two fp16 terms:
 *                        u < 2048 keeps 22 significant bits (what makes the selected experts agree with an fp32
 *                        reference except on near-ties), 2048 <= u <= 65504 keeps 11, larger u saturates;
 *       router layer 2   Wr2 is used as fp16: its bf16 values convert exactly when |Wr2| is in [6.2e-5, 65504] or 0
 *                        (smaller magnitudes lose bits to fp16's subnormal range).
 *     With unit-variance activations and weights of the usual initialisations all of these hold with orders of
 *     magnitude to spare; activations that are not normalised may need SLICEMOE_FLAG_FORCE_GENERIC (fp32 arithmetic).
 *   - Errors are return codes; nothing aborts or throws across this boundary.
 */
#ifndef SLICEMOE_H
#define SLICEMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    SLICEMOE_OK = 0,
    SLICEMOE_ERR_INVALID_ARG = 1, /* null pointer, non-positive size, d % S != 0, k > E ...   */
    SLICEMOE_ERR_UNSUPPORTED = 2, /* valid layer, but outside the limits listed above          */
    SLICEMOE_ERR_WORKSPACE = 3,   /* workspace / packed buffer too small                       */
    SLICEMOE_ERR_HIP = 4          /* a kernel launch reported an error (hipGetLastError)       */
} slicemoe_status;

typedef enum { SLICEMOE_F32 = 0, SLICEMOE_BF16 = 1 } slicemoe_dtype;

/* flags */
#define SLICEMOE_FLAG_FORCE_GENERIC 1u /* never use the MFMA kernels (debug / cross-check)      */
#define SLICEMOE_FLAG_REQUIRE_MFMA 2u  /* return UNSUPPORTED instead of using generic kernels   */
#define SLICEMOE_FLAG_SINGLE_STREAM 4u /* slicemoe_backward keeps every kernel on `stream`      */

/* Same handle type as hipStream_t, spelled out so this header needs no HIP include. */
struct ihipStream_t;
typedef struct ihipStream_t *slicemoe_stream_t;

typedef struct {
    int32_t T;  /* tokens                                                                   */
    int32_t d;  /* token width                                                              */
    int32_t S;  /* slices per token (Section 3)                                             */
    int32_t k;  /* experts per slice (Section 3.1)                                          */
    int32_t E;  /* experts                                                                  */
    int32_t Hr; /* router hidden width (256 in the paper, Section 3.1 / Appendix A)         */
    int32_t He; /* expert hidden width                                                      */
    float capacity_factor; /* <= 0: dropless.  > 0: per-expert row capacity
                              C = ceil((double)capacity_factor * T*S*k / E); within an expert
                              rows are ranked by ascending slice id and rank >= C is dropped
                              (contributes zero to h').                                      */
    int32_t dtype; /* slicemoe_dtype                                                        */
    uint32_t flags;
} slicemoe_config;

/* Layer parameters, logical layout.  `packed` is optional (NULL allowed): the buffer
 * written by slicemoe_pack_weights for the same config and tensors.  When it is NULL and a
 * kernel wants the packed form, the call packs into its workspace first (slower). */
typedef struct {
    const void *Wr1; /* [ds, Hr]   router layer 1 */
    const void *br1; /* [Hr]                      */
    const void *Wr2; /* [Hr, E]    router layer 2 */
    const void *br2; /* [E]                       */
    const void *W1;  /* [E, ds, He] expert layer 1 */
    const void *b1;  /* [E, He]                    */
    const void *W2;  /* [E, He, ds] expert layer 2 */
    const void *b2;  /* [E, ds]                    */
    const void *packed;
} slicemoe_weights;

/* Byte offsets of the intermediates that slicemoe_forward leaves in its workspace. */
typedef struct {
    size_t topk_idx;   /* int32 [T*S, k]                                   */
    size_t topk_p;     /* float [T*S, k]                                   */
    size_t counts_raw; /* int32 [E]                                        */
    size_t counts;     /* int32 [E]                                        */
    size_t offsets;    /* int32 [E+1]                                      */
    size_t perm;       /* int32 [T*S*k]                                    */
    size_t inv;        /* int32 [T*S*k]                                    */
    size_t y;          /* float or fp16 [T*S*k, ds] (see dtype above)      */
    size_t stats;      /* float [4], see slicemoe_load_stats               */
    size_t scratch;    /* dispatch scratch                                 */
    size_t packed;     /* on-the-fly packed weights                        */
    size_t total;      /* == slicemoe_workspace_bytes                      */
} slicemoe_workspace_layout;

const char *slicemoe_status_string(slicemoe_status s);

/* 1 if this config would run on the MFMA kernels, 0 if on the generic ones, -1 if invalid. */
int slicemoe_uses_mfma(const slicemoe_config *cfg);

/* Per-expert capacity C for this config, or -1 when dropless / invalid. */
int64_t slicemoe_capacity(const slicemoe_config *cfg);

/* Workspace sizes in bytes (0 on an invalid or unsupported config).  The forward workspace
 * also satisfies slicemoe_dispatch.  Workspaces must be 256-byte aligned. */
size_t slicemoe_workspace_bytes(const slicemoe_config *cfg);
size_t slicemoe_dispatch_workspace_bytes(const slicemoe_config *cfg);
slicemoe_status slicemoe_get_workspace_layout(const slicemoe_config *cfg, slicemoe_workspace_layout *out);

/* One-time re-tiling of the weights into matrix-core fragment order (a weight-load step,
 * like any layout transform done when a model is loaded; Section 3.4 leaves the kernel's
 * internals open).  packed_bytes is 0 when the config runs on the generic kernels; then
 * slicemoe_pack_weights is a no-op returning OK. */
size_t slicemoe_packed_bytes(const slicemoe_config *cfg);
slicemoe_status slicemoe_pack_weights(const slicemoe_config *cfg, const slicemoe_weights *w,
                                      void *packed_out, size_t packed_bytes, slicemoe_stream_t stream);

/*
 * Router (Section 3.1): for every slice, logits g = ReLU(x Wr1 + br1) Wr2 + br2, p = softmax(g)
 * over all E experts (temperature 1, not renormalised over the selected k), top-k on the fp32
 * logits, equal logits resolved to the lower expert index, slot 0 = largest.
 *   h        [T, d]    in
 *   topk_idx [T*S, k]  out int32
 *   topk_p   [T*S, k]  out float, p of each selected expert
 *   workspace: needed only when w->packed is NULL on the MFMA path (>= slicemoe_workspace_bytes);
 *              may be NULL otherwise.
 */
slicemoe_status slicemoe_route(const slicemoe_config *cfg, const void *h, const slicemoe_weights *w,
                               int32_t *topk_idx, float *topk_p,
                               void *workspace, size_t workspace_bytes, slicemoe_stream_t stream);

/*
 * Training-time router: slicemoe_route with the variations the paper describes around it, applied in the order
 * logits -> noise -> top-k and softmax -> dropout.
 *   temperature  tau > 0 (Appendix B; default 1): p = softmax(g / tau).  The selection does not depend on it.
 *   noise_std    sigma >= 0 (Section 5, robustness to router noise): g <- g + sigma * noise[n, e] before the
 *                softmax, hence also before the selection.
 *   dropout_rate r in [0, 1) (Section 3.3, cross-slice dropout; Appendix A uses 0.2): selected assignment j of slice
 *                n is dropped when drop_u[n, j] < r; the slice's remaining probabilities are renormalised to sum to 1
 *                and the dropped ones become 0; if all k would drop, slot 0 is kept.  With r > 0 every slice is
 *                renormalised.  topk_idx keeps all k experts: a dropped assignment stays assigned with probability
 *                0, so by Eq. 1 its expert sees the zero vector.
 * The random draws are INPUTS, so a run is reproducible from its arguments alone:
 *   noise  [T*S, E] float, standard-normal draws, 16-byte aligned; read only when noise_std > 0 (may be NULL otherwise)
 *   drop_u [T*S, k] float, uniform draws in [0, 1); read only when dropout_rate > 0 (may be NULL otherwise)
 * Other arguments, layouts and workspace as slicemoe_route.  INVALID_ARG for params == NULL, a parameter outside its
 * range (or NaN / infinite), or a table the parameters need that is NULL or misaligned.
 */
typedef struct {
    float temperature;
    float noise_std;
    float dropout_rate;
    float capacity_alpha;   /* read by slicemoe_backward only (see there); 0 = the capacity loss sends no gradient */
} slicemoe_route_train_params;
slicemoe_status slicemoe_route_train(const slicemoe_config *cfg, const void *h, const slicemoe_weights *w,
                                     const slicemoe_route_train_params *params, const float *noise,
                                     const float *drop_u, int32_t *topk_idx, float *topk_p,
                                     void *workspace, size_t workspace_bytes, slicemoe_stream_t stream);

/*
 * Dispatch (the grouping of Section 3.4): stable counting sort of assignments by expert.
 *   topk_idx   [T*S, k] in, values in [0, E) (out-of-range values are clamped, never faulted on)
 *   counts_raw [E]      out: assignments per expert (the counts of Eq. 2)
 *   counts     [E]      out: min(counts_raw, C)
 *   offsets    [E+1]    out: exclusive scan of counts; offsets[E] = number of kept rows
 *   perm       [T*S*k]  out: perm[row] = assignment id of stacked row `row` (rows of one expert
 *                            are contiguous, in ascending slice order); entries at
 *                            row >= offsets[E] are left untouched
 *   inv        [T*S*k]  out: inv[a] = row of assignment a, or -1 if it was dropped
 *   workspace  >= slicemoe_dispatch_workspace_bytes
 */
slicemoe_status slicemoe_dispatch(const slicemoe_config *cfg, const int32_t *topk_idx,
                                  int32_t *counts_raw, int32_t *counts, int32_t *offsets,
                                  int32_t *perm, int32_t *inv,
                                  void *workspace, size_t workspace_bytes, slicemoe_stream_t stream);

/*
 * slicemoe_dispatch for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid allocation.  Same arguments, outputs and bits as
 * slicemoe_dispatch, minus the workspace: the per-chunk histogram table lives in a fixed 1 MiB array inside the
 * library's device image (one copy per GPU, held until the process ends).  The call allocates and frees nothing.
 *   Limit: the table, E rows of ceil(T*S*k / chunk) entries (rounded up to a multiple of 8; chunk = 1024 assignments
 *   while that gives at most 4096 chunks, else 2048, else 4096), must fit 262144 entries: any config with
 *   T*S*k <= 16 777 216.  Beyond it the call returns SLICEMOE_ERR_WORKSPACE and launches nothing.
 *   All calls on one GPU share the array: calls that overlap in time on one GPU (different streams) race on it.
 *   Nothing in it has to be cleared between calls; it keeps the last call's table.
 */
slicemoe_status slicemoe_dispatch_noalloc(const slicemoe_config *cfg, const int32_t *topk_idx,
                                          int32_t *counts_raw, int32_t *counts, int32_t *offsets,
                                          int32_t *perm, int32_t *inv, slicemoe_stream_t stream);

/*
 * Expert FFN on the stacked batch (Eq. 1, Section 3.1 expert, Section 3.4 grouping): for every
 * kept row r < offsets[E], with a = perm[r], n = a / k and e the expert whose range holds r,
 *   y[r, :] = GELU((topk_p[a] * x[n, :]) W1[e] + b1[e]) W2[e] + b2[e]
 * The gather of x and the Eq. 1 weighting are fused into the kernel (no stacked copy of the
 * inputs is materialised); the He-wide hidden activations never leave the chip.
 *   y [T*S*k, ds] out, fp32 (fp32 storage) or fp16 (bf16 storage); rows >= offsets[E] are left untouched.
 * The MFMA kernel evaluates GELU(z) = z Phi(z) in packed fp16 with a polynomial for Phi and feeds
 * fp16 hidden activations to its second GEMM (activation error of the size of one bf16 rounding,
 * hidden activations beyond +-2.6e5 would overflow); the generic kernel uses erf in fp32.
 */
slicemoe_status slicemoe_expert_ffn(const slicemoe_config *cfg, const void *h, const float *topk_p,
                                    const int32_t *offsets, const int32_t *perm,
                                    const slicemoe_weights *w, void *y,
                                    void *workspace, size_t workspace_bytes, slicemoe_stream_t stream);

/*
 * Combine (Section 3.1): h'[n, :] = sum over the kept assignments j of slice n of
 * y[inv[n*k + j], :] (fp32 or fp16, as above), summed in fp32 in ascending j, rounded once to the storage dtype and
 * written at h_out[t, s*ds : (s+1)*ds].  A slice with all k assignments dropped gives zeros.
 */
slicemoe_status slicemoe_combine(const slicemoe_config *cfg, const void *y, const int32_t *inv,
                                 void *h_out, slicemoe_stream_t stream);

/*
 * Load statistics of a routed batch, computed on device from the dispatch counts:
 *   stats[0] = CV^2 of counts_raw with the population variance (= L_cap / alpha, Eq. 2)
 *   stats[1] = ELE = -sum_e load_e log(load_e) / log(E), load_e = counts_raw[e] / sum (Section 4)
 *   stats[2] = dropped fraction 1 - sum(counts) / sum(counts_raw)
 *   stats[3] = CV^2 with the sample variance (E-1 in the denominator)
 */
slicemoe_status slicemoe_load_stats(const slicemoe_config *cfg, const int32_t *counts_raw,
                                    const int32_t *counts, float *stats, slicemoe_stream_t stream);

/*
 * Whole layer: h[T, d] -> h_out[T, d] = route, dispatch, expert FFN, combine, load stats, all on
 * `stream`.  Intermediates stay in `workspace` at the offsets of slicemoe_get_workspace_layout.
 */
slicemoe_status slicemoe_forward(const slicemoe_config *cfg, const void *h, const slicemoe_weights *w,
                                 void *h_out, void *workspace, size_t workspace_bytes,
                                 slicemoe_stream_t stream);

/*
 * Whole layer with the training-time router: slicemoe_forward with slicemoe_route_train in place of slicemoe_route
 * (same parameters and tables of draws); dispatch, expert FFN (Eq. 1 with the dropped-and-renormalised probabilities)
 * and combine are unchanged.
 */
slicemoe_status slicemoe_forward_train(const slicemoe_config *cfg, const void *h, const slicemoe_weights *w,
                                       const slicemoe_route_train_params *params, const float *noise,
                                       const float *drop_u, void *h_out, void *workspace, size_t workspace_bytes,
                                       slicemoe_stream_t stream);

/*
 * Backward pass of the layer: gradients of a scalar loss that depends on h and on the weights only through h', by
 * the chain rule through the sum over the k experts, the expert FFN and the Eq. 1 input weighting (Section 3.1) and
 * the router (Section 3.1; temperature of Appendix B, logit noise of Section 5, cross-slice dropout of Section 3.3).
 * The routing decisions -- which experts a slice selected, which assignments the capacity limit dropped, which the
 * dropout zeroed -- are piecewise constant and held fixed.  The router receives gradient through the selected
 * probabilities, which weight the expert inputs (z = p (x W1) + b1, so dL/dp = sum over the hidden units of
 * dL/dz (x W1)); with dropout the renormalisation is differentiated; the noise is an additive constant.
 * The capacity loss (Section 3.2, Eq. 2) is a function of integer counts and has zero gradient as written, although
 * Section 3.1 trains the router with it; its value is alpha * stats[0] of slicemoe_load_stats.  With
 * params->capacity_alpha = alpha != 0 this call adds the gradient of a differentiable stand-in, the usual one for a
 * count-based balance loss: the count of expert e is replaced by the sum c_e of the final probabilities (topk_p, after
 * dropout) of the assignments routed to e, the loss by alpha * CV^2(c_1..c_E) with the population variance, so that
 * dL_cap/dp_a = alpha (2E / S^2) (c_e(a) - Q / S) with S = sum c, Q = sum c^2 is added to dL/dp of every assignment,
 * also of those the capacity limit dropped (they still count as assigned); it reaches the router's weights and dL/dh.
 * The sums are accumulated as 64-bit integers (p * 2^38), so this term too is the same bits on every run.
 *   h, w                 as given to the forward call (w: the LOGICAL tensors are read, w->packed is ignored)
 *   params, noise, drop_u as given to slicemoe_forward_train; params == NULL after slicemoe_forward
 *   forward_workspace    the workspace that forward call filled (routing tables and probabilities are read from it)
 *   d_out [T, d] in      dL/dh', storage dtype
 *   d_h   [T, d] out     dL/dh, storage dtype (one rounding)
 *   grads       out      one fp32 DEVICE array per weight tensor, logical layout, overwritten.  Partial sums are
 *                        added in a fixed order: same inputs, bit-identical weight gradients and dL/dh, on every
 *                        path (no floating-point atomics anywhere in the backward).
 *   workspace            >= slicemoe_backward_workspace_bytes(cfg), 256-byte aligned
 *   stream               the call's place in this stream orders it against the caller's other work, as for every entry
 *                        point.  On the matrix-core path the expert weight gradients (one kernel and its reduction,
 *                        which the rest of the backward neither feeds nor needs) run on a second stream that the library
 *                        owns (one per device, default priority, created at the first backward on the device and kept
 *                        until the process ends): it is forked from `stream` after the weights are repacked and joined
 *                        back into `stream` before the call returns, so everything the call writes is complete when the
 *                        work the caller enqueues next on `stream` runs.  The pattern is a plain fork and join with two
 *                        events, which a HIP graph capture of `stream` takes along (after one eager call has created
 *                        the stream).  Calls from several host threads on one device are enqueued one after the other.
 *                        SLICEMOE_FLAG_SINGLE_STREAM keeps every kernel on `stream` (same results, a few percent slower).
 * For bf16 storage with d/S in {64, 96, 128} and He % 32 == 0 (slicemoe_backward_uses_mfma: 1, 0, or -1 for an
 * invalid config) the expert part (row gradients, dL/dp, expert weight gradients) runs on the matrix cores, and with
 * Hr = 256 the router part too: fp32 pre-activations and derivatives, two-term bf16 operands
 * for the second matrix instructions, fp32-grade results.  Everything else runs on vector-ALU kernels in fp32.
 * SLICEMOE_FLAG_FORCE_GENERIC selects those throughout.  UNSUPPORTED for Hr > 256.
 */
typedef struct {
    float *Wr1, *br1, *Wr2, *br2, *W1, *b1, *W2, *b2;
} slicemoe_weight_grads;
int slicemoe_backward_uses_mfma(const slicemoe_config *cfg);
size_t slicemoe_backward_workspace_bytes(const slicemoe_config *cfg);
slicemoe_status slicemoe_backward(const slicemoe_config *cfg, const void *h, const slicemoe_weights *w,
                                  const slicemoe_route_train_params *params, const float *noise, const float *drop_u,
                                  const void *forward_workspace, size_t forward_workspace_bytes,
                                  const void *d_out, void *d_h, const slicemoe_weight_grads *grads,
                                  void *workspace, size_t workspace_bytes, slicemoe_stream_t stream);

#ifdef __cplusplus
}
#endif
#endif /* SLICEMOE_H */
