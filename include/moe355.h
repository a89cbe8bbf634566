/*
 * moe355.h -- C ABI of libmoe355: one Mixture-of-Experts layer with top-k gating,
 * forward and backward, on one AMD MI355X (gfx950).
 *
 * What the layer computes is Algorithm 1 of the FastMoE paper ("Forward computation
 * of an MoE layer with top-k gating") for every row x of X:
 *
 *     score = G(x);  indices = ArgMax_k(score);  y = sum_{i in indices} score_i * E_i(x)
 *
 * with the notation of the paper's Section 5.1: n_b = N input samples, n_e = E experts
 * (all on this GPU), each expert two linear layers of sizes d_m x d_h and d_h x d_m
 * (d and h here), top-k selection.  The gate G is one fully-connected layer (Section
 * 5.2).  How it is computed is the reordering of the paper's Section 4: the samples
 * of one expert are placed in a contiguous buffer ("scatter"), each expert processes
 * its batch as matrix products, and the rows are put back in their original order
 * ("gather"); the per-expert sample counts are taken first and fix the buffer layout
 * (Section 3.2, description of the global operations figure).
 *
 * Points on which the paper is silent and this library fixes a reading:
 *   logits l = x W_g + b_g;  top-k on the logits, equal logits -> lower expert id,
 *   slot j = j-th largest;  score = softmax over the k selected logits;
 *   E_e(x) = GeLU(x W1[e] + b1[e]) W2[e] + b2[e] with the erf GeLU (the biases are optional);
 *   inside an expert's segment rows keep assignment order a = t*k + j;
 *   backward = gradient of <dY, Y> with the selected indices held constant.
 *
 * All matrices are dense row-major.  Every pointer named "device" must be device
 * memory of the current HIP device, 16-byte aligned, owned by the caller for the
 * whole call and until the stream work has completed.  The library allocates no
 * device memory and keeps no pointer after a call returns.  Its state, all of it
 * behind locks: the thread-local error string; per device, which kernels have had
 * their LDS limit raised and the device's compute-unit count (filled in on first
 * use); the event pool of the optional per-kernel timing (moe_profile_*: the one
 * place that creates HIP events); the 16 MiB device array of
 * moe_scatter_backward_static.  All work is enqueued on `stream` (a hipStream_t
 * passed as void*, NULL = the null stream); no call synchronises with the host or
 * copies anything to the host, except moe_check_status and moe_profile_read, which
 * say so.  Calls return a status; nothing throws or aborts.
 * The calls enqueue kernels only (no memset or copy nodes), so a sequence of them
 * may be captured in a HIP graph once each has run once on the device outside a
 * capture (the first launch of some kernels sets a function attribute); replays
 * give the bits of the eager run (while per-kernel timing is off: moe_profile_*).
 */
#ifndef MOE355_H
#define MOE355_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOE_OK = 0,
    MOE_ERR_INVALID_ARG = -1, /* null required pointer, misaligned pointer, N<0, k<1, k>E, ...  */
    MOE_ERR_UNSUPPORTED = -2, /* d or h not a multiple of 32, E>1024, k>8, unknown dtype,
                                 non-zero reserved field, score_all with the standalone
                                 backward calls                                              */
    MOE_ERR_WORKSPACE = -3,   /* workspace smaller than moe_workspace_bytes()                 */
    MOE_ERR_HIP = -4          /* a kernel launch (or its set-up: a function attribute, a device
                                 query) reported an error; moe_last_error() has the text      */
} moe_status_t;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype_t;

/* Problem description; plain host struct passed by pointer. */
typedef struct {
    int32_t N;          /* n_b: rows of X (tokens); 0 is allowed (nothing is launched)        */
    int32_t d;          /* d_m: model width, multiple of 32                                   */
    int32_t h;          /* d_h: expert hidden width, multiple of 32                           */
    int32_t E;          /* n_e: experts, 1..1024                                              */
    int32_t k;          /* experts selected per token, 1..min(E,8)                            */
    int32_t dtype;      /* moe_dtype_t of X, W_g, W1, W2, Y, dY, dX and the saved activations */
    int32_t grad_dtype; /* moe_dtype_t of dW1, dW2, dW_g: equal to dtype, or MOE_F32          */
    int32_t accumulate; /* 0: weight gradients are overwritten (zeros for an expert that got
                           no row); 1: added to what the buffers hold                         */
    int32_t score_all;  /* 0: the scores of a token are the softmax over its k selected logits
                           (they sum to 1); 1: the softmax over all E logits, taken at the
                           selected experts (Algorithm 1 read literally with a softmax gate:
                           they sum to less than 1, and every expert's gate column, selected or
                           not, receives gradient - also with k = 1)                           */
    int32_t balance_stats; /* 1: moe_plan keeps what moe_balance_stats needs (the gate logits) in the
                           workspace; implied by score_all                                     */
    int32_t reserved[6]; /* must be zero                                                      */
} moe_desc_t;

/* Routing of one batch; six caller-owned device arrays that moe_plan fills and
 * moe_forward / moe_backward read.  M = N*k assignments, a = t*k + j. */
typedef struct {
    int32_t *topk_idx; /* [N,k] expert of slot j of token t, slots in descending logit order  */
    float *topk_w;     /* [N,k] combine weight (score) of that slot; a row sums to 1 (less than
                          1 with desc->score_all)                                            */
    int32_t *counts;   /* [E]   rows received by each expert                                  */
    int32_t *offsets;  /* [E+1] exclusive prefix sum of counts; offsets[E] = M                */
    int32_t *pos;      /* [M]   assignment a -> row of the expert-contiguous buffers          */
    int32_t *perm;     /* [M]   row of the expert-contiguous buffers -> assignment a          */
} moe_plan_t;

/* Bytes of device workspace the three calls below need for this problem (expert-contiguous
 * activations Xs, Z, H, Ys, their gradients, the tile schedule, reduction scratch and, for bf16,
 * 64 MiB in which the matrix-product workgroups hand partial sums to one another).
 * Returns 0 if desc is NULL or not supported. Host-only; touches no device. */
size_t moe_workspace_bytes(const moe_desc_t *desc);

/*
 * Gate, selection, counting and layout (Algorithm 1 steps "score" and "indices"; the
 * count / offset step of Section 3.2).
 *   X  device [N,d] dtype;  Wg device [d,E] dtype;  bg device [E] float or NULL (= zeros).
 *   plan: host struct holding six device arrays, all written.
 *   workspace: device, >= moe_workspace_bytes(); the tile schedule written here (and the flags
 *   and status word cleared here) are used by moe_forward / moe_backward, which must receive the
 *   same workspace.  Calls that share a workspace must not overlap in time.
 * The selection is exact: logits are accumulated in fp64, so indices, counts and the
 * permutation are those of exact arithmetic unless two logits agree to ~1e-15 relative.
 */
moe_status_t moe_plan(const moe_desc_t *desc, const void *X, const void *Wg, const float *bg,
                      moe_plan_t *plan, void *workspace, size_t workspace_bytes, void *stream);

/*
 * Forward: scatter, per-expert FFN as grouped matrix products, weighted gather
 * (Section 4 reordering of Algorithm 1's loop).
 *   W1 device [E,d,h], W2 device [E,h,d] dtype.
 *   b1 device [E,h], b2 device [E,d] dtype, or NULL: the biases of the expert's two linear
 *   layers (the paper's expert is an FFN, Section 5.1): E_e(x) = GeLU(x W1[e] + b1[e]) W2[e] + b2[e].
 *   Y device [N,d] dtype, written.
 * Leaves Z (pre-activation), H and Ys in the workspace for moe_backward.  bf16: Z is the
 * rounded accumulator, H = z * Phi(Z) with z the fp32 accumulator and Phi the normal CDF taken at
 * the stored Z (the erf GeLU up to that rounding inside Phi, which moves H by less than 6e-4).
 * The two data movements of Section 4 are done on the fly where that saves a pass over memory: the
 * first layer reads row perm[r] / k of X as row r of its input (no scattered copy is written in the
 * forward pass; moe_backward writes Xs for the weight gradients), and with k = 1 and score_all = 0,
 * where y is the one selected expert's output, the second layer writes its rows straight to their
 * tokens' rows of Y (then no Ys is kept, and none is needed: the gate receives no gradient).
 */
moe_status_t moe_forward(const moe_desc_t *desc, const moe_plan_t *plan, const void *X, const void *W1,
                         const void *W2, const void *b1, const void *b2, void *Y, void *workspace,
                         size_t workspace_bytes, void *stream);

/*
 * Backward of L = <dY, Y> (the paper states that forward and backward both run through
 * the same reordering, Section 3.2, and that the gate is trained through the score,
 * Section 2.1).  Must follow moe_forward on the same desc, plan and untouched workspace.
 *   dY device [N,d] dtype.
 *   dX device [N,d] dtype, written (expert path + gate path).
 *   dWg device [d,E], dW1 device [E,d,h], dW2 device [E,h,d] in grad_dtype; written or
 *   accumulated per desc->accumulate.  dbg device [E] float or NULL, same rule.
 * Weight gradients are reduced in a fixed order: repeated calls give identical bits.
 */
moe_status_t moe_backward(const moe_desc_t *desc, const moe_plan_t *plan, const void *X, const void *Wg,
                          const void *W1, const void *W2, const void *dY, void *dX, void *dWg, float *dbg,
                          void *dW1, void *dW2, void *workspace, size_t workspace_bytes, void *stream);

/*
 * The status word of a workspace, copied to the host: 0, or 1 if since the last moe_plan on this workspace a
 * grouped-product workgroup's bounded wait for another workgroup's partial sum ran out (then the results of those
 * calls are invalid and moe_last_error() says so).  The persistent grouped-product kernels hand partial sums from
 * one workgroup to the next and assume that all of a launch's workgroups (one per compute unit) are resident
 * together, which holds when nothing else occupies the GPU's compute units for long; a caller that runs other
 * kernels beside these on other streams should check the word.
 * WAITS for the work enqueued on `stream` and copies 4 bytes to the host (one of the two calls that synchronise).
 *   status: host int32, written.
 */
moe_status_t moe_check_status(const moe_desc_t *desc, const void *workspace, size_t workspace_bytes, void *stream,
                              int32_t *status);

/*
 * Load-balance monitor of the batch routed by the last moe_plan on this workspace (the paper leaves
 * a load-balance monitor to future work, Section 6; these are the statistics one is built from).
 * Needs desc->balance_stats or desc->score_all.
 *   fraction  device [E] float: counts[e] / (N k), the share of the assignments expert e received
 *   mean_prob device [E] float: mean over the tokens of softmax(x W_g + b_g)[e]
 *   loss      device [1] float: E * sum_e fraction[e] mean_prob[e]  (1 for a gate that cannot tell
 *             the experts apart, E when one expert gets everything with certainty); any may be NULL.
 * Sums run in a fixed order.  With N == 0 the outputs are zeros.
 */
moe_status_t moe_balance_stats(const moe_desc_t *desc, const moe_plan_t *plan, float *fraction,
                               float *mean_prob, float *loss, void *workspace, size_t workspace_bytes,
                               void *stream);

/*
 * Gradients of the expert biases (only needed when moe_forward was given b1 / b2; the other
 * gradients do not change form with biases, since Z is stored with b1 included).  Must follow
 * moe_backward on the same desc, plan and untouched workspace: per expert it sums, in a fixed
 * order, the rows of dZ (db1) and of the weighted output gradients dYs (db2) that moe_backward
 * left there.
 *   db1 device [E,h] float or NULL, db2 device [E,d] float or NULL; written, or added to when
 *   desc->accumulate is 1.  Rows of experts that received no token are zero (or unchanged).
 */
moe_status_t moe_bias_backward(const moe_desc_t *desc, const moe_plan_t *plan, float *db1, float *db2,
                               void *workspace, size_t workspace_bytes, void *stream);

/*
 * The data-movement steps on their own, so that any expert network can sit between them (the
 * paper's layer takes an arbitrary expert module: Section 3.1; the reordering itself is Section 4,
 * "scatter" before the experts and "gather" after them).  All four take a plan written by moe_plan
 * for the same desc (desc->h is not used) and caller-owned buffers in the expert-contiguous row
 * order of the plan: row pos[a] belongs to assignment a = t*k + j, rows of expert e are
 * offsets[e] .. offsets[e+1]-1.  M = N*k.  Same status codes and stream rules as above.
 *
 *   moe_scatter:          Xs[pos[a],:] = X[a / k,:]                    X [N,d] -> Xs [M,d] (copy)
 *   moe_gather:           Y[t,:] = sum_j topk_w[t,j] * Ys[pos[t*k+j],:]   Ys [M,d] -> Y [N,d]
 *                         (slots in ascending order, fp32 accumulation)
 *   moe_gather_backward:  dYs[pos[a],:] = topk_w[a] * dY[t,:]  and the gradient of the selected logits,
 *                         dl[t,j] = w_j (dw_j - sum_i w_i dw_i) with dw_j = <dY[t,:], Ys[pos[t*k+j],:]>
 *                         (the weights are a softmax over the k selected logits; exact zeros for k = 1).
 *                         dY [N,d], Ys [M,d] -> dYs [M,d] dtype, dl [M] float in assignment order.
 *   moe_scatter_backward: dX[t,:] = sum_j dXs[pos[t*k+j],:] + sum_j dl[t,j] * Wg[:,idx[t,j]]   (expert path
 *                         + gate path), dWg[:,e] (+)= sum over assignments of e of dl * x, dbg likewise.
 *                         Wg [d,E], Xs [M,d] (as written by moe_scatter), dXs [M,d], dl [M] -> dX [N,d] dtype,
 *                         dWg [d,E] grad_dtype and dbg [E] float (or NULL), written or accumulated per
 *                         desc->accumulate.  Needs the workspace that moe_plan wrote for this plan (it reads the table of
 *                         64-row pieces there and keeps its fixed-order reduction there).
 * With N == 0 nothing is launched except that moe_scatter_backward still writes dWg / dbg (zeros, or
 * leaves them when accumulating).
 */
moe_status_t moe_scatter(const moe_desc_t *desc, const moe_plan_t *plan, const void *X, void *Xs, void *stream);
moe_status_t moe_gather(const moe_desc_t *desc, const moe_plan_t *plan, const void *Ys, void *Y, void *stream);
moe_status_t moe_gather_backward(const moe_desc_t *desc, const moe_plan_t *plan, const void *dY, const void *Ys,
                                 void *dYs, float *dl, void *stream);
moe_status_t moe_scatter_backward(const moe_desc_t *desc, const moe_plan_t *plan, const void *Wg, const void *Xs,
                                  const void *dXs, const float *dl, void *dX, void *dWg, float *dbg,
                                  void *workspace, size_t workspace_bytes, void *stream);

/*
 * moe_scatter_backward for callers that cannot allocate device memory or carry a workspace: code under HIP
 * graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments (minus the workspace),
 * same kernels and the same bits as moe_scatter_backward.  What that call keeps in the workspace (the table of
 * 64-row pieces, the fp32 partial sums of the gate-matrix gradient by piece, the transposed gate matrix) lives
 * in a device array of 16 MiB that is part of the library's code object: every GPU the library runs on holds
 * its own copy until the process ends.  The call allocates and frees nothing (no hipMalloc, no hipFree, no
 * allocating library routine); its first call on a device looks the array's address up.
 *   Limit: (N k / 64 + E) (4 d + 4) + E d sizeof(dtype) + 16 (E + 1) bytes, each part rounded up to 256, must
 *   fit in 16 MiB (all five benchmark workloads do); larger problems return MOE_ERR_WORKSPACE with the sizes in
 *   moe_last_error() and must use moe_scatter_backward.
 *   All calls on one GPU share that GPU's array, which keeps the last call's contents (nothing in it has to
 *   start at zero: every word a kernel reads was written earlier in the same call).  Calls that overlap in time
 *   on one GPU (different streams, different threads) race on it: the caller serialises them.
 *   Unlike moe_scatter_backward it does not read the workspace that moe_plan wrote, only the plan arrays.
 */
moe_status_t moe_scatter_backward_static(const moe_desc_t *desc, const moe_plan_t *plan, const void *Wg, const void *Xs,
                                         const void *dXs, const float *dl, void *dX, void *dWg, float *dbg,
                                         void *stream);

/*
 * Where a named intermediate lives inside the workspace (host-only; touches no device).
 * Names: "Z" [M,h] pre-activations, "H" [M,h] GeLU(Z), "Ys" [M,d]
 * expert outputs before the weighted gather (valid after moe_forward; "Ys" not with k = 1 and
 * score_all = 0); "Xs" [M,d] scattered inputs, "dYs" [M,d], "dZ" [M,h], "dXs" [M,d] (dtype elements)
 * and "dl" [M] float, the gradient of the selected logits (valid after moe_backward).  Rows are in expert-contiguous order (row r holds
 * assignment perm[r]).  "gate_uncertified": [1 + N] int32, valid after moe_plan
 * for bf16 with 17 to 256 experts (score_all = balance_stats = 0): how many tokens the gate kernel that ranks
 * fp32 logits could not settle within its error bound (more than 16 candidates for the k places, or no finite bound) and
 * handed to the kernel that evaluates every logit in fp64, then their ids in no particular order.  "status": the int32 that
 * moe_check_status returns.  "clock": two int64 written by the last bf16 matrix-product launch,
 * shader cycles and ticks of the 100 MHz reference clock over the lifetime of one of its workgroups
 * (their ratio x 100 is the shader clock in MHz the launch ran at).  Returns MOE_ERR_INVALID_ARG for an
 * unknown name.
 */
moe_status_t moe_workspace_region(const moe_desc_t *desc, const char *name, size_t *offset, size_t *bytes);

/*
 * Diagnostics: per-kernel timing with HIP events, off by default (the one stateful, allocating corner of the
 * library: a process-wide switch and a pool of events behind a mutex).  While enabled, every kernel
 * group the three calls launch is bracketed by two events recorded on the caller's stream (this
 * creates events, the one place where the library allocates, and adds a few microseconds per
 * launch, so whole-step timings should be taken with it disabled).
 *   moe_profile_enable(on)  switches it on (1) or off (0); switching discards pending records.
 *   moe_profile_read(out, max)  WAITS for the recorded events (the only call that synchronises
 *     with the device), writes up to `max` entries -- one per kernel group, with the number of
 *     launches and their summed duration since the last read -- and returns how many it wrote
 *     (negative status on a HIP error).  `name` points to static storage.
 */
typedef struct {
    const char *name; /* e.g. "ggemm_fc1_gelu", "scatter"; "ggemm_dxs+dw1" is one launch that   */
                      /* holds two grouped products                                             */
    int32_t launches; /* launches recorded since the last read                                  */
    double total_ms;  /* summed device time of those launches                                   */
} moe_kernel_time_t;
moe_status_t moe_profile_enable(int on);
int moe_profile_read(moe_kernel_time_t *out, int max_entries);

/* Text of the last error on this thread ("" if none). Static storage; do not free. */
const char *moe_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* MOE355_H */
