/*
 * moe.h -- C ABI of the MI355X (gfx950) library for one GPU's share of a TED
 * Mixture-of-Experts layer: top-1 gate, capacity-limited routing, dispatch into
 * per-expert buffers, the per-expert FFN shard (GEMM, GeLU, GEMM), the
 * gate-weighted combine, and the backward of all of these; plus the tiled optimizer
 * step for the expert parameters (last entry point).
 *
 * Paper: "A Hybrid Tensor-Expert-Data Parallelism Approach to Optimize
 * Mixture-of-Experts Training" (DeepSpeed-TED).  The layer is Section 1 /
 * Figure 1 (a routing function sends each token to exactly one expert FFN);
 * the per-GPU order of work is Section 3, Figure 3, steps 3 (routing), 4 (tokens
 * leave for their expert), 5 (expert FFN, one tensor-parallel partition), 7
 * (tokens return); the backward runs the same steps in reverse (end of
 * Section 3).  This library is the local computation between the collectives:
 * steps 2, 4, 6 and 7's communication is not part of it, so the FFN output is
 * the partial sum of this GPU's f inner columns.
 *
 * Notation: T tokens, h hidden size, E experts, f FFN inner width owned by this
 * GPU (4h / G_tensor), C capacity (rows per expert buffer), e_t / s_t / p_t the
 * expert, slot and gate probability of token t, kept_e = min(count_e, C).
 *
 * Conventions for every entry point
 *  - All array arguments are DEVICE pointers (HBM) unless marked "host".
 *    All arrays are dense, row-major, with the index order written next to them,
 *    and must be 16-byte aligned.  The caller owns every buffer; the library
 *    never allocates, frees or keeps a pointer after the call returns.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls
 *    only enqueue work on it; there is no host synchronisation and no host read
 *    of device data (kept_e is read on the device, so launches cover C rows per
 *    expert and skip the unused part).  One exception to "only on `stream`":
 *    moe_expert_ffn_bwd (bf16) runs its two weight-gradient GEMMs on an internal
 *    stream that starts behind an event of `stream`, and `stream` waits for that stream's last
 *    event before the call's work is complete, so the caller still orders everything
 *    on `stream` alone.  One internal stream (and three events) exists per caller stream and device,
 *    created on first use and kept until the process ends; calls on different streams do not share
 *    one.  Two host threads must not call moe_expert_ffn_bwd on the SAME stream at once (they would
 *    interleave on it anyway).  Beyond 8 caller streams per device, and always when MOE_TED_SERIAL=1
 *    is set before the first call, everything stays on `stream`.
 *  - `dtype` is the storage type of x, buffers, expert weights and their
 *    gradients: MOE_BF16 (fp32 accumulation on MFMA) or MOE_F32.  The gate
 *    (w_gate, logits, probs, gate_p and their gradients) is always fp32.
 *  - Returns MOE_OK or an error code; never throws or aborts.  Arguments are
 *    validated on the host before anything is launched: a failed call launches
 *    nothing.  moe_last_error() gives a thread-local description.
 *  - Not checked (undefined results, no memory fault as long as the arrays have
 *    the stated sizes and expert/slot came from moe_gate): non-finite logits.
 *  - Limits: 1 <= E <= 256; h and f multiples of 8 (bf16) or 4 (fp32), at most
 *    2^20; 1 <= T, C < 2^31; T*h*sizeof(dtype) < 2^37; E*C*max(h,f) < 2^40;
 *    C*max(h,f)*sizeof(dtype) < 2^31 and h*f*sizeof(dtype) < 2^31 (one expert's
 *    chunk and one expert's weight matrix are addressed through 32-bit
 *    windows; whole tensors may be larger than 4 GiB).
 */
#ifndef MOE_TED_H
#define MOE_TED_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    MOE_OK = 0,
    MOE_ERR_INVALID_ARG = 1,        /* null pointer, non-positive size, misaligned pointer */
    MOE_ERR_UNSUPPORTED = 2,        /* size outside the limits above, unknown dtype/act */
    MOE_ERR_WORKSPACE_TOO_SMALL = 3,
    MOE_ERR_HIP = 4                 /* a HIP launch reported an error */
} moe_status_t;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1 } moe_dtype_t;
typedef enum { MOE_GELU_ERF = 0, MOE_GELU_TANH = 1 } moe_act_t;

typedef struct {
    int64_t T;      /* tokens on this GPU */
    int32_t h;      /* hidden size */
    int32_t E;      /* experts */
    int32_t f;      /* FFN inner width of this tensor-parallel shard */
    int64_t C;      /* capacity: rows per expert buffer */
    int32_t dtype;  /* moe_dtype_t */
    int32_t act;    /* moe_act_t */
} moe_shape_t;

/* Host helpers (pure, no GPU needed). */

/* C = ceil(capacity_factor * T / E) evaluated in double; 0 on bad arguments. */
int64_t moe_capacity(int64_t T, int32_t E, double capacity_factor);

/* Bytes of device workspace the calls below need for this shape (one workspace serves
 * all calls of a layer; contents need not survive between calls).
 * for_backward: 0 = forward only, 1 = forward and backward, 2 = forward and backward with
 * activation recomputation (moe_expert_ffn_fwd called with hact = NULL, moe_expert_ffn_bwd with
 * hact = z_save = NULL).  0 on a bad shape or mode. */
size_t moe_workspace_bytes(const moe_shape_t *shape, int for_backward);

const char *moe_status_string(moe_status_t s);
const char *moe_last_error(void);   /* thread-local text of the last failure in this thread */
int moe_version(void);

/*
 * Measurement aid: enqueues n (0..4096) empty one-wave kernels on `stream`, back to back.  The routing
 * kernels move a few hundred KB and are bound by launch latency, not by HBM (their cost is quoted in
 * microseconds); this is the floor those microseconds are read against: the time the GPU needs per
 * dependent launch when a kernel does nothing.  Nothing is read or written.
 */
moe_status_t moe_launch_floor(int32_t n, void *stream);

/*
 * Gate + routing (Section 3, step 3: the routing function runs on every GPU over the tokens that
 * GPU holds; Section 1: the function is parameterised and maps each token to exactly one expert).
 *   logits[t,j] = sum_k x[t,k] w_gate[k,j]  (+ logit_bias[j])      fp32
 *   e_t   = lowest j attaining max_j logits[t,j]
 *   probs = softmax_j(logits[t,:]),  p_t = probs[t,e_t]
 *   s_t   = #{u < t : e_u = e_t};  slot[t] = s_t if s_t < C else -1 (dropped)
 *   counts[e] = #{t : e_t = e} (before dropping);  kept[e] = min(counts[e], C)
 *   token_of_slot[e,s] = the token holding slot s of expert e, -1 if the slot is empty
 * x == NULL: `logits` is an input (already biased) and w_gate / logit_bias are ignored;
 * otherwise `logits` is an output.  probs may be NULL when no backward follows.
 *   x [T,h] dtype, w_gate [h,E] f32, logit_bias [E] f32 or NULL, logits [T,E] f32,
 *   probs [T,E] f32 or NULL, expert [T] i32, gate_p [T] f32, slot [T] i32,
 *   counts [E] i32, kept [E] i32, token_of_slot [E,C] i32.
 * Routing outputs are integers and are reproducible bit for bit (no dependence on
 * atomic ordering).
 */
moe_status_t moe_gate(const moe_shape_t *shape, const void *x, const float *w_gate, const float *logit_bias,
                      float *logits, float *probs, int32_t *expert, float *gate_p, int32_t *slot,
                      int32_t *counts, int32_t *kept, int32_t *token_of_slot, void *ws, size_t ws_bytes,
                      void *stream);

/*
 * Dispatch (Section 3, step 4, local half: tokens are grouped by destination expert into
 * equal-size chunks, which is the send layout of the all-to-all).
 *   buf[e,s,:] = x[token_of_slot[e,s],:]  for filled slots (s < kept[e]).
 * Empty slots (s >= kept[e]) are NOT written: the padding of an expert's chunk carries no
 * information, nothing in this library reads it (every later step takes kept[e] rows), and
 * filling it would add up to (capacity_factor - 1) / capacity_factor of the step's HBM writes.
 * After a call, rows kept[e] .. C-1 of expert e hold whatever they held before (an earlier step's
 * tokens when kept[e] has shrunk, not zeros).  A caller that ships whole C-row chunks to another
 * GPU therefore either sends kept[e] along with chunk e, or clears rows kept[e] .. C-1 itself in
 * every step; clearing buf once at allocation is not enough.  The same holds for the unwritten rows
 * of y, d_y and d_buf.
 *   x [T,h], token_of_slot [E,C], buf [E,C,h].
 */
moe_status_t moe_dispatch(const moe_shape_t *shape, const void *x, const int32_t *token_of_slot, void *buf,
                          void *stream);

/*
 * Expert FFN forward (Section 3, step 5; Section 2.4: a pair of consecutive fully connected
 * layers, of which this GPU holds f inner columns of the first and the matching f rows of the
 * second, so y is a partial sum that step 6's all-reduce would complete).
 *   for r < kept[e]:  z = buf[e,r,:] w1[e] ;  hact = GeLU(z) ;  y[e,r,:] = hact w2[e]
 * Rows r >= kept[e] of hact, z_save and y are not written.
 *   buf [E,C,h], w1 [E,h,f], w2 [E,f,h], kept [E], y [E,C,h],
 *   hact [E,C,f] (out; the backward needs it) or NULL: GeLU(z) then lives in the workspace only,
 *   z_save [E,C,f] or NULL (out, needed by backward: it receives GeLU'(z), the only function of
 *   the pre-activation the backward pass uses, so that backward does not evaluate erf again).
 * hact = z_save = NULL is the forward of a layer trained with activation recomputation (the paper
 * trains with activation checkpointing throughout, Section 5): between forward and backward only
 * buf, y and the routing arrays are held; moe_expert_ffn_bwd recomputes the rest.
 * Workspace: the tile plans of the two GEMMs (bf16), plus E*C*f*sizeof(dtype) when hact is NULL.
 */
moe_status_t moe_expert_ffn_fwd(const moe_shape_t *shape, const void *buf, const void *w1, const void *w2,
                                const int32_t *kept, void *z_save, void *hact, void *y, void *ws,
                                size_t ws_bytes, void *stream);

/*
 * moe_expert_ffn_fwd for callers that cannot allocate or size a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same computation, same kernels and
 * bit-identical results; the only scratch of the call, the tile plans of its two GEMMs (fetch counters
 * and tile queues), lives in an array inside the library's device image instead of a caller workspace.
 * The call allocates and frees nothing (no hipMalloc, no hipFree, no allocating library routine).
 *  - hact must be given (without a workspace there is nowhere else to keep GeLU(z)); z_save may be NULL.
 *  - Limit: the two plans must fit MOE_STATIC_SCRATCH_BYTES; a plan takes
 *    128 + 16 * E * ceil(C / 256) * ceil(N / 256) bytes (N = f for the first GEMM, h for the second),
 *    rounded up to 256.  Larger shapes return MOE_ERR_UNSUPPORTED (nothing is launched) and must use
 *    moe_expert_ffn_fwd.
 *    The 6.7B-base shard (E=16, C=1280, h=f=4096) needs 41 KB.
 *  - Each GPU holds one such array for the life of the process and every call on that GPU uses it:
 *    two calls that overlap on one GPU (different streams, or different host threads) race on the
 *    plans and give undefined results; calls ordered on one stream are fine.  The array keeps the
 *    previous call's contents; the call rewrites every word it reads before the GEMMs start.
 *  - The array's device address is looked up on the first call on each device (not an allocation);
 *    make that first call outside stream capture.
 */
#define MOE_STATIC_SCRATCH_BYTES (256u * 1024u)
moe_status_t moe_expert_ffn_fwd_static(const moe_shape_t *shape, const void *buf, const void *w1, const void *w2,
                                       const int32_t *kept, void *z_save, void *hact, void *y, void *stream);

/*
 * Combine (Section 3, step 7, local half: tokens come back to their original position; the
 * gate probability weights the expert's output).
 *   out[t,:] = gate_p[t] * y[expert[t], slot[t], :]  if slot[t] >= 0, else 0.
 *   y [E,C,h], expert [T], slot [T], gate_p [T], out [T,h].
 */
moe_status_t moe_combine(const moe_shape_t *shape, const void *y, const int32_t *expert, const int32_t *slot,
                         const float *gate_p, void *out, void *stream);

/*
 * Dispatch, expert FFN forward and combine in one call (Section 3, local halves of steps 4, 5 and 7):
 *   out[t,:] = gate_p[t] * ( GeLU(x[t,:] w1[e_t]) w2[e_t] )   for kept tokens, 0 for dropped ones,
 * with the two row permutations folded into the GEMMs: the first GEMM takes the rows of expert e
 * straight from x through token_of_slot[e,:] (no dispatch buffer is written or read), and the second
 * GEMM's epilogue writes every result row, times its token's gate probability, to that token's row of
 * out.  bf16 only.  The results (out, and hact / z_save / y where given) are bit-identical to
 * moe_dispatch + moe_expert_ffn_fwd + moe_combine.
 *   x [T,h] or NULL, buf [E,C,h] or NULL: exactly one of the two (buf: rows already dispatched, as a
 *   training step needs them anyway for the weight gradient; x: gathered, T*h*2 < 2^31),
 *   token_of_slot [E,C], slot [T], gate_p [T], w1 [E,h,f], w2 [E,f,h], kept [E],
 *   z_save [E,C,f] or NULL, hact [E,C,f] or NULL, y [E,C,h] or NULL (the backward needs y), out [T,h].
 * Workspace: moe_workspace_bytes (any mode) suffices: tile plans, E*C floats, and hact when it is NULL.
 */
moe_status_t moe_expert_ffn_fwd_fused(const moe_shape_t *shape, const void *x, const void *buf,
                                      const int32_t *token_of_slot, const int32_t *slot, const float *gate_p,
                                      const void *w1, const void *w2, const int32_t *kept, void *z_save, void *hact,
                                      void *y, void *out, void *ws, size_t ws_bytes, void *stream);

/* ---- duplicate token dropping (Section 5.1, Figure 5), the local halves ----
 *
 * The G = tp_size GPUs of a tensor-parallel group hold identical expert chunks before the first
 * all-to-all.  Each performs a "drop" that leaves it a share of the rows, disjoint from the other
 * ranks' shares, so the all-to-all messages shrink by the factor G; after the all-to-all an all-gather
 * inside the group reassembles the chunks.  In the backward pass the two steps change places.  The paper
 * does not fix which rows a rank keeps; this library's convention: rank r keeps rows s with s mod G = r
 * of every expert chunk, in order, so row s of a chunk is row s / G of share s mod G.  A share is
 * [E, Cg, h] with Cg = ceil(C / G); shares of all ranks, as the all-gather delivers them, are
 * [G, E, Cg, h].  Rows that correspond to empty slots (s >= kept[e]) are never written and never read.
 * Requirements for all five calls: 1 <= tp_size <= C, 0 <= tp_rank < tp_size.
 */

/*
 * Dispatch fused with the drop of rank tp_rank (Figure 5, step 1, on top of Section 3, step 4):
 *   share[e, j, :] = x[token_of_slot[e, j * tp_size + tp_rank], :]   for filled slots.
 *   x [T,h], token_of_slot [E,C], share [E,Cg,h] (out).
 */
moe_status_t moe_dispatch_dtd(const moe_shape_t *shape, const void *x, const int32_t *token_of_slot, int32_t tp_rank,
                              int32_t tp_size, void *share, void *stream);

/*
 * The drop alone, for any [E,C,h] row array (the backward pass drops d_buf before the reverse all-to-all):
 *   share[e, j, :] = buf[e, j * tp_size + tp_rank, :]   for j * tp_size + tp_rank < kept[e].
 */
moe_status_t moe_dtd_drop(const moe_shape_t *shape, const void *buf, const int32_t *kept, int32_t tp_rank,
                          int32_t tp_size, void *share, void *stream);

/*
 * The all-gathered shares put back in row order (Figure 5, step 2, local half), as a copy:
 *   buf[e, s, :] = shares[s mod tp_size][e, s / tp_size, :]   for s < kept[e].
 * A training step needs this array (the weight gradient reads the dispatched rows along its reduction
 * index); a forward-only layer does not: moe_expert_ffn_fwd_dtd reads the shares in place.
 *   shares [G,E,Cg,h], kept [E], buf [E,C,h] (out).
 */
moe_status_t moe_dtd_gather(const moe_shape_t *shape, const void *shares, const int32_t *kept, int32_t tp_size,
                            void *buf, void *stream);

/*
 * moe_expert_ffn_fwd whose first GEMM takes row s of expert e straight from shares[s mod G][e, s / G, :]
 * (the strided form of the gathered operand load of moe_expert_ffn_fwd_fused): no reassembled copy of the
 * chunks is written or read.  bf16 only; G*E*Cg*h*2 < 2^31.  Results are bit-identical to
 * moe_dtd_gather + moe_expert_ffn_fwd.  Other arguments and workspace as for moe_expert_ffn_fwd.
 */
moe_status_t moe_expert_ffn_fwd_dtd(const moe_shape_t *shape, const void *shares, int32_t tp_size, const void *w1,
                                    const void *w2, const int32_t *kept, void *z_save, void *hact, void *y, void *ws,
                                    size_t ws_bytes, void *stream);

/*
 * moe_dispatch_bwd reading the all-gathered gradient shares (backward of Figure 5: the drop of d_buf by
 * moe_dtd_drop, the reverse all-to-all, then an all-gather) in place:
 *   d_x[t,:] = d_shares[slot[t] mod G][expert[t], slot[t] / G, :] if slot[t] >= 0 else 0   (+ d_logits[t,:] w_gate^T).
 *   d_shares [G,E,Cg,h]; the other arguments as for moe_dispatch_bwd.
 */
moe_status_t moe_dispatch_bwd_dtd(const moe_shape_t *shape, const void *d_shares, int32_t tp_size,
                                  const int32_t *expert, const int32_t *slot, void *d_x, const float *d_logits,
                                  const float *w_gate, void *stream);

/* ---- backward (end of Section 3: the same steps in reverse order) ---- */

/*
 * Combine backward.
 *   d_y[e_t,s_t,:] = gate_p[t] * d_out[t,:] ;  d_gate_p[t] = <d_out[t,:], y[e_t,s_t,:]>
 *   for kept tokens; d_gate_p[t] = 0 for dropped tokens; empty slots of d_y (s >= kept[e]) are
 *   not written (moe_expert_ffn_bwd reads kept[e] rows per expert).
 *   d_out [T,h], y [E,C,h], token_of_slot [E,C], gate_p [T], d_y [E,C,h], d_gate_p [T] f32.
 */
moe_status_t moe_combine_bwd(const moe_shape_t *shape, const void *d_out, const void *y,
                             const int32_t *token_of_slot, const int32_t *slot, const float *gate_p, void *d_y,
                             float *d_gate_p, void *stream);

/*
 * Expert FFN backward.
 *   d_h = d_y w2[e]^T ;  d_z = d_h * z_save  (z_save = GeLU'(z) from the forward) ;  d_w2[e] = hact^T d_y ;
 *   d_w1[e] = buf^T d_z ;  d_buf = d_z w1[e]^T          (rows r < kept[e] only)
 * d_w1, d_w2 are overwritten (one micro-batch), in `dtype` with fp32 accumulation; an expert
 * with kept[e] = 0 gets zero gradients.  Rows r >= kept[e] of d_buf are not written.
 * z_save = hact = NULL (both or neither): activation recomputation -- the forward's first GEMM is run
 * again from buf and w1 and writes hact and GeLU'(z) into the workspace, then the backward proceeds
 * as above; the results are bit-identical to the stored-activation call.
 * Uses E*C*f*sizeof(dtype) bytes of workspace for d_z, plus (bf16) the tile plans of the GEMMs, plus
 * 2*E*C*f*sizeof(dtype) when recomputing (moe_workspace_bytes(shape, 2)).
 */
moe_status_t moe_expert_ffn_bwd(const moe_shape_t *shape, const void *d_y, const void *buf, const void *z_save,
                                const void *hact, const void *w1, const void *w2, const int32_t *kept,
                                void *d_buf, void *d_w1, void *d_w2, void *ws, size_t ws_bytes, void *stream);

/*
 * Dispatch backward:  d_x[t,:] = d_buf[expert[t], slot[t], :] if slot[t] >= 0 else 0.
 * If d_logits and w_gate are given (both or neither), the gate's contribution to the token gradient
 * is added in the same pass:  d_x[t,:] += d_logits[t,:] w_gate^T  (d_logits from moe_gate_bwd), so
 * d_x is written once.
 *   d_buf [E,C,h], expert [T], slot [T], d_x [T,h] (out), d_logits [T,E] f32 or NULL,
 *   w_gate [h,E] f32 or NULL.
 */
moe_status_t moe_dispatch_bwd(const moe_shape_t *shape, const void *d_buf, const int32_t *expert,
                              const int32_t *slot, void *d_x, const float *d_logits, const float *w_gate,
                              void *stream);

/*
 * Gate backward (the gate only receives gradient through p_t).
 *   d_logits[t,j] = d_gate_p[t] * p_t * ([j == e_t] - probs[t,j])
 *   d_w_gate = x^T d_logits ;  d_x_accum[t,:] += d_logits[t,:] w_gate^T   (if d_x_accum != NULL; the
 *   same term can instead be fused into moe_dispatch_bwd, which is the cheaper order:
 *   moe_combine_bwd, moe_gate_bwd(d_x_accum = NULL), moe_expert_ffn_bwd, moe_dispatch_bwd(d_logits, w_gate))
 *   d_gate_p [T] f32, probs [T,E] f32, expert [T], x [T,h], w_gate [h,E] f32,
 *   d_logits [T,E] f32 (out), d_w_gate [h,E] f32 (out, overwritten) or NULL,
 *   d_x_accum [T,h] dtype (in/out) or NULL.
 */
moe_status_t moe_gate_bwd(const moe_shape_t *shape, const float *d_gate_p, const float *probs,
                          const int32_t *expert, const void *x, const float *w_gate, float *d_logits,
                          float *d_w_gate, void *d_x_accum, void *ws, size_t ws_bytes, void *stream);

/*
 * Tiled mixed-precision AdamW step for a flat group of n expert parameters.
 * Paper, Section 4: before the update the optimizer up-casts the 16-bit gradients to 32 bit; for the
 * expert parameter group that temporary is 4 bytes per parameter, so the group is cut into tiles of
 * ts parameters, processed one after the other, and one temporary of 4*ts bytes serves every tile
 * (the paper fixes ts = 1.8 million).  The optimizer is AdamW (Section 6, set-up).
 * Per parameter i, with t = hp->step >= 1:
 *   g   = fp32(grad[i]) * hp->grad_mult               (the up-cast; grad_mult = inverse loss scale, 1 = none)
 *   m   = beta1 m + (1 - beta1) g ;   v = beta2 v + (1 - beta2) g^2
 *   w   = w - lr * ( (m / (1 - beta1^t)) / (sqrt(v / (1 - beta2^t)) + eps) + weight_decay * w )
 *   param[i] = dtype(w)                                (round to nearest even for bf16)
 * evaluated in fp32; master, exp_avg, exp_avg_sq are updated in place.
 *   grad [n] dtype, master [n] f32 (in/out), exp_avg [n] f32 (in/out), exp_avg_sq [n] f32 (in/out),
 *   param [n] dtype (out), hp: host pointer, read before the call returns.
 *   staging: [min(ts, n)] f32 device buffer, the ONLY temporary of the step, contents undefined
 *   afterwards; for each tile the up-cast gradients are written there and the update reads them.
 *   staging == NULL: the up-cast happens in registers inside the update, no temporary exists and ts
 *   is ignored.  Both ways, and every ts, give bit-identical results.
 * With a staging buffer and ts < n, ts must be a multiple of 8.  n = 0 is a no-op.
 * Errors: MOE_ERR_INVALID_ARG for NULL / misaligned arrays, ts < 1, step < 1, beta outside [0, 1),
 * negative or non-finite lr, eps, weight_decay; MOE_ERR_UNSUPPORTED for n >= 2^40, a ts that is not a
 * multiple of 8, or an unknown dtype.
 */
typedef struct {
    float lr, beta1, beta2, eps, weight_decay;
    float grad_mult;   /* multiplies every gradient during the up-cast */
    int32_t step;      /* t: 1 for the first update */
} moe_adamw_t;

moe_status_t moe_adamw_tiled(int64_t n, int64_t ts, const moe_adamw_t *hp, const void *grad, float *master,
                             float *exp_avg, float *exp_avg_sq, void *param, float *staging, int32_t dtype,
                             void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_TED_H */
