/*
 * flexmoe.h -- C ABI of the single-GPU FlexMoE MoE-layer hot path for AMD MI355X (gfx950).
 *
 * The layer one GPU executes under a dynamic vExpert placement (arXiv 2304.03946):
 *   gate top-k (Eq. 3) -> route: split every expert's tokens evenly over its vExperts
 *   (Section 3.2, Alg. 3 with a single GPU) -> permute into contiguous per-vExpert buckets
 *   (Section 4, expert-wise layout transformation) -> expert FFN per bucket (Eq. 2, forward
 *   and backward, which is what the cost T_C of Eq. 7 covers) -> un-permute and gate-weighted
 *   sum (Eq. 4).
 *
 * Conventions shared by every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller, row-major, contiguous,
 *     16-byte aligned.  The only HOST pointers are the placement table arguments of
 *     flexmoe_route (rep_off_host, rep_ids_host).
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only
 *     enqueue work; they never allocate, free or synchronise, and the library keeps no state
 *     between calls (tables it needs are constant data of the code object).  Scratch memory comes
 *     from the caller: `ws` with at least flexmoe_workspace_bytes(...) bytes, 256-byte aligned.
 *     An entry point may overwrite all of `ws`; its contents mean nothing to the next call, with one
 *     stated exception: flexmoe_expert_ffn_bwd (and _bwd_top1) leaves dHpre at the start of `ws`,
 *     where flexmoe_expert_bias_grads reads it when called next with the same `ws`.
 *   - Arguments are validated on the host before anything is launched; on an error nothing
 *     is written.  Return value: a flexmoe_status code.
 *   - Notation: N tokens, d = d_model, f = d_ff, E experts, k experts per token, V vExperts,
 *     A = N*k assignments.  Assignment id a = t*k + j (token t, j-th choice of its gate).
 *   - dtype selects the element type of x, weights, activations and outputs (gate weights are
 *     always float, indices always int32).  BF16 computes with bf16 MFMA and fp32
 *     accumulation; F32 computes in fp32.  d and f must be multiples of 8.
 *   - Limits: E <= 256, V <= 512, k <= 8, A < 2^30.
 */
#ifndef FLEXMOE_H
#define FLEXMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FLEXMOE_MAX_EXPERTS 256
#define FLEXMOE_MAX_VEXPERTS 512
#define FLEXMOE_MAX_TOPK 8

enum flexmoe_status {
  FLEXMOE_OK = 0,
  FLEXMOE_INVALID_ARG = 1,         /* null pointer, negative or out-of-range size, misaligned d/f */
  FLEXMOE_BAD_PLACEMENT = 2,       /* table is not a partition of 0..V-1 with >=1 vExpert per expert */
  FLEXMOE_WORKSPACE_TOO_SMALL = 3,
  FLEXMOE_UNSUPPORTED = 4,         /* unknown dtype or activation */
  FLEXMOE_DEVICE_ERROR = 5,        /* a kernel launch failed */
  FLEXMOE_SCRATCH_LIMIT = 6        /* flexmoe_route_static: the problem needs more than its fixed scratch */
};

enum flexmoe_dtype { FLEXMOE_F32 = 0, FLEXMOE_BF16 = 1 };
enum flexmoe_act { FLEXMOE_RELU = 0, FLEXMOE_GELU_ERF = 1, FLEXMOE_GELU_TANH = 2 };

/* Human-readable name of a status code (static storage). */
const char* flexmoe_status_str(int status);

/* Bytes of scratch that any entry point may need for the given problem (max over all). */
size_t flexmoe_workspace_bytes(int N, int d, int f, int E, int k, int V, int dtype);

/*
 * Top-k gate, Eq. 3:  l = x . W_g ;  keep the k largest logits of each token; softmax over
 * the kept ones.
 *   x [N,d] dtype, wg [d,E] dtype  ->  topk_idx [N,k] int32, topk_w [N,k] float.
 * Slot j holds the j-th largest logit; equal logits order by lower expert id.  Logits are
 * accumulated in fp32.  NaN inputs give unspecified selections.
 */
int flexmoe_gate_topk(const void* x, const void* wg, int N, int d, int E, int k, int dtype,
                      int32_t* topk_idx, float* topk_w, void* ws, size_t ws_bytes, void* stream);

/*
 * Router, Section 3.2 (vExperts: each replicates exactly one expert; an expert's tokens are
 * partitioned evenly over its vExperts) and Alg. 3 with one GPU (everything stays local).
 *   topk_idx [N,k] int32 (device), values in [0,E)
 *   rep_off_host [E+1], rep_ids_host [V]  (HOST, CSR): the vExperts of expert e are
 *       rep_ids_host[rep_off_host[e] .. rep_off_host[e+1]), in replica order.
 * Outputs (device, int32):
 *   expert_count [E]    I_e, assignments per expert
 *   vexpert_count [V]   share of each vExpert: floor(I_e/n_e), +1 for the first I_e mod n_e replicas
 *   vexpert_off [V+1]   exclusive prefix sum of vexpert_count in ascending vExpert id
 *   vexpert_owner [V]   the expert each vExpert replicates
 *   dest [A]            bucket slot of assignment a: an expert's assignments, in ascending a,
 *                       are cut into contiguous chunks, one per replica in list order
 *   src [A]             inverse permutation, src[dest[a]] = a
 * Results do not depend on scheduling (no atomics-ordered ranks): two calls give identical bits.
 */
int flexmoe_route(const int32_t* topk_idx, int N, int k, int E, int V,
                  const int32_t* rep_off_host, const int32_t* rep_ids_host,
                  int32_t* expert_count, int32_t* vexpert_count, int32_t* vexpert_off,
                  int32_t* vexpert_owner, int32_t* dest, int32_t* src,
                  void* ws, size_t ws_bytes, void* stream);

/*
 * Expert-wise layout transformation (Section 4): gather tokens into the per-vExpert buckets.
 *   xp[p,:] = x[src[p] / k, :] * (row_scale ? row_scale[src[p]] : 1)      p in [0,A)
 *   x [N,d] dtype, src [A], row_scale [A] float indexed by assignment id or NULL -> xp [A,d] dtype.
 * With row_scale = topk_w this is also the backward of flexmoe_combine w.r.t. its input.
 */
int flexmoe_permute(const void* x, const int32_t* src, const float* row_scale,
                    int N, int k, int d, int dtype, void* xp, void* stream);

/*
 * Expert FFN forward, Eq. 2 in row-vector form, per bucket v owned by expert e:
 *   hpre[rows_v,:] = xp[rows_v,:] . W1_e + b1_e ;  yp[rows_v,:] = act(hpre[rows_v,:]) . W2_e + b2_e
 *   xp [A,d], w1 [E,d,f], b1 [E,f] or NULL, w2 [E,f,d], b2 [E,d] or NULL, all dtype;
 *   vexpert_off [V+1], vexpert_owner [V] as written by flexmoe_route.
 *   -> hpre [A,f] dtype (pre-activation, kept for the backward pass), yp [A,d] dtype.
 *   hpre may be NULL when no backward pass follows (inference): the pre-activations are then not
 *   stored, which halves what the first product writes; yp is the same, bit for bit.
 *   h [A,f] dtype or NULL: where act(hpre), the second product's operand, is written.  NULL keeps it in
 *   the workspace (gone after the call).  A caller that hands the same buffer to the backward pass saves
 *   that pass computing and storing it again (the backward's first kernel then writes one [A,f] tensor
 *   instead of two); the price is A*f more elements of saved activations per layer.  Same bits either way.
 * The activation is applied to hpre as stored (i.e. after rounding to dtype).
 */
int flexmoe_expert_ffn_fwd(const void* xp, const int32_t* vexpert_off, const int32_t* vexpert_owner,
                           const void* w1, const void* b1, const void* w2, const void* b2,
                           int A, int d, int f, int E, int V, int act, int dtype,
                           void* hpre, void* h, void* yp, void* ws, size_t ws_bytes, void* stream);

/*
 * Expert FFN backward (the backward half of T_C, Eq. 7) for upstream gradient dyp [A,d]:
 *   dH = dyp . W2_e^T ; dHpre = dH * act'(hpre) ; dxp = dHpre . W1_e^T
 *   dw2[e] = sum over the vExperts v of e of act(hpre_v)^T . dyp_v      [E,f,d]
 *   dw1[e] = sum over the vExperts v of e of xp_v^T . dHpre_v           [E,d,f]
 * The sum over an expert's vExperts is the on-chip image of the replica gradient
 * synchronisation (T_Sync, Eq. 9); it runs in ascending vExpert id with fp32 accumulation.
 * dw1/dw2 are overwritten (not accumulated); experts without tokens get zeros.
 *   h [A,f] dtype or NULL: act(hpre) as a forward call left it in its `h` argument.  NULL: it is computed
 *   again from hpre (into the workspace).  Same results, bit for bit.
 */
int flexmoe_expert_ffn_bwd(const void* dyp, const void* xp, const void* hpre, const void* h,
                           const void* w1, const void* w2,
                           const int32_t* vexpert_off, const int32_t* vexpert_owner,
                           int A, int d, int f, int E, int V, int act, int dtype,
                           void* dxp, void* dw1, void* dw2, void* ws, size_t ws_bytes, void* stream);

/*
 * flexmoe_expert_ffn_bwd for a top-1 layer (k = 1) with the backward reverse routing folded in: bucket
 * row p of dXp is stored as row src[p] of dx, i.e. dx [N,d] is the expert-path gradient of the layer
 * input and flexmoe_combine(dxp, dest, NULL) is not needed (same bits).  dw1, dw2 as in
 * flexmoe_expert_ffn_bwd; the workspace afterwards serves flexmoe_expert_bias_grads in the same way.
 *   src [N] as written by flexmoe_route with k = 1; h as in flexmoe_expert_ffn_bwd.
 * FLEXMOE_UNSUPPORTED unless dtype is bf16 and f is a multiple of 128.
 */
int flexmoe_expert_ffn_bwd_top1(const void* dyp, const void* xp, const void* hpre, const void* h,
                                const void* w1, const void* w2,
                                const int32_t* vexpert_off, const int32_t* vexpert_owner, const int32_t* src,
                                int N, int d, int f, int E, int V, int act, int dtype,
                                void* dx, void* dw1, void* dw2, void* ws, size_t ws_bytes, void* stream);

/*
 * Reverse routing and gate-weighted sum, Eq. 4:
 *   y[t,:] = sum_j (topk_w ? topk_w[t*k+j] : 1) * yp[dest[t*k+j], :]
 *   yp [A,d] dtype, dest [A], topk_w [N,k] float or NULL -> y [N,d] dtype (fp32 accumulation).
 * With topk_w = NULL this is the backward of flexmoe_permute w.r.t. x.
 */
int flexmoe_combine(const void* yp, const int32_t* dest, const float* topk_w,
                    int N, int k, int d, int dtype, void* y, void* stream);

/*
 * flexmoe_permute followed by flexmoe_expert_ffn_fwd without materialising xp: bucket row p of the
 * first product is read as row src[p] / k of x while the tile is loaded (Section 4's layout
 * transformation folded into the expert computation).  Same results as the two calls, bit for bit.
 *   x [N,d], src [A] (A = N*k) as written by flexmoe_route; everything else as in
 *   flexmoe_expert_ffn_fwd (hpre and h may be NULL as well).  For forward-only use: the backward pass reads xp.
 * FLEXMOE_UNSUPPORTED unless dtype is bf16, d is a multiple of 128 and N*d < 2^30: callers then
 * use the two separate calls.
 */
int flexmoe_expert_ffn_fwd_gather(const void* x, const int32_t* src, const int32_t* vexpert_off,
                                  const int32_t* vexpert_owner, const void* w1, const void* b1,
                                  const void* w2, const void* b2,
                                  int N, int k, int d, int f, int E, int V, int act, int dtype,
                                  void* hpre, void* h, void* yp, void* ws, size_t ws_bytes, void* stream);

/*
 * The expert path of a top-1 layer (k = 1) in one call, without xp and yp: bucket row p is read as row
 * src[p] of x while the first product's tiles are loaded, and the second product's rows are stored
 * straight to y[src[p], :] (Section 4's layout transformation and the reverse routing of Eq. 4 folded
 * into the expert computation; with one expert per token the gate value is exactly 1).  Same y as
 * flexmoe_permute + flexmoe_expert_ffn_fwd + flexmoe_combine, bit for bit.
 *   x [N,d], src [N] as written by flexmoe_route with k = 1 -> hpre [N,f], h [N,f] (each may be NULL), y [N,d].
 * For forward-only use.  FLEXMOE_UNSUPPORTED unless dtype is bf16, d and f are multiples of 128 and
 * N*d < 2^30.
 */
int flexmoe_expert_ffn_fwd_top1(const void* x, const int32_t* src, const int32_t* vexpert_off,
                                const int32_t* vexpert_owner, const void* w1, const void* b1,
                                const void* w2, const void* b2,
                                int N, int d, int f, int E, int V, int act, int dtype,
                                void* hpre, void* h, void* y, void* ws, size_t ws_bytes, void* stream);

/*
 * Backward of the gate path (Eq. 3-4; the logits are x . W_g, the top-k kept, softmax over the
 * kept ones) for an upstream gradient dy of the layer output.  Completes a trainable layer
 * together with flexmoe_expert_ffn_bwd, which treats the gate values as constants.
 *   dg[t,j] = <dy[t,:], yp[dest[t*k+j],:]>        yp: the experts' outputs in bucket order (forward)
 *   dl[t,j] = topk_w[t,j] * (dg[t,j] - sum_i topk_w[t,i] * dg[t,i])      -> dl [N,k] float
 *   dx[t,:] += sum_j dl[t,j] * wg[:, topk_idx[t,j]]     dx [N,d] dtype, IN/OUT: holds the expert-path
 *                                                       gradient on entry (flexmoe_combine of dxp)
 *   dwg[:,e] = sum over the assignments a routed to e of dl[a] * x[a div k,:]   -> dwg [d,E] dtype,
 *              overwritten; summed over xp (= flexmoe_permute of x) bucket by bucket in a fixed order
 *   wg [d,E], dy [N,d], yp [A,d], xp [A,d] dtype; topk_idx/topk_w [N,k]; dest/src [A];
 *   vexpert_off [V+1], vexpert_owner [V] as written by flexmoe_route.
 * With k = 1 the single kept gate value is 1 whatever the logit: dl and dwg are zero, dx unchanged.
 */
int flexmoe_gate_bwd(const void* wg, const int32_t* topk_idx, const float* topk_w, const void* dy,
                     const void* yp, const void* xp, const int32_t* dest, const int32_t* src,
                     const int32_t* vexpert_off, const int32_t* vexpert_owner,
                     int N, int d, int E, int k, int V, int dtype,
                     float* dl, void* dx, void* dwg, void* ws, size_t ws_bytes, void* stream);

/*
 * Bias gradients of Eq. 2: db1_e = sum of the rows of dHpre in e's buckets, db2_e = the same for
 * dyp (the gate-scaled, permuted upstream gradient that flexmoe_expert_ffn_bwd consumed).
 *   db1 [E,f], db2 [E,d] dtype, overwritten (zeros for experts without tokens); either may be NULL.
 * `ws` must be the workspace of the preceding flexmoe_expert_ffn_bwd call of the same sizes,
 * untouched since (the one place where a workspace carries data from call to call, see the
 * conventions above): dHpre [A,f] is read from its start, and the part behind dHpre is overwritten.
 * Fixed summation order: reproducible bit for bit.
 */
int flexmoe_expert_bias_grads(const void* dyp, const int32_t* vexpert_off, const int32_t* vexpert_owner,
                              int A, int d, int f, int E, int V, int dtype,
                              void* db1, void* db2, void* ws, size_t ws_bytes, void* stream);

/*
 * flexmoe_route for callers that cannot allocate device memory or hand over a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus
 * ws / ws_bytes), same kernels, same results bit for bit.  The scratch (per-unit expert histograms)
 * is a fixed array of FLEXMOE_ROUTE_STATIC_SCRATCH_BYTES inside the library, one copy per GPU, held
 * until the process ends; its address is looked up on the first call on each device.  Allocates
 * nothing, frees nothing, does not synchronise.
 *   Limit: units * E * 4 <= FLEXMOE_ROUTE_STATIC_SCRATCH_BYTES, where units = ceil(A / 256) for
 *   A <= 65536, ceil(A / 512) up to A = 524288, at most 1024 beyond; e.g. any A with E <= 64, and
 *   A <= 65536 with E = 256.  Larger problems return FLEXMOE_SCRATCH_LIMIT and launch nothing.
 *   All calls on one GPU share the array: calls that overlap in time on one GPU (different
 *   streams, or graphs replayed concurrently) race and must be serialised by the caller.  Nothing in
 *   the array has to start at zero (every entry that is read is written first by the same call).
 */
#define FLEXMOE_ROUTE_STATIC_SCRATCH_BYTES (256 * 1024)
int flexmoe_route_static(const int32_t* topk_idx, int N, int k, int E, int V,
                         const int32_t* rep_off_host, const int32_t* rep_ids_host,
                         int32_t* expert_count, int32_t* vexpert_count, int32_t* vexpert_off,
                         int32_t* vexpert_owner, int32_t* dest, int32_t* src, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* FLEXMOE_H */
