/*
 * lazarus_moe.h -- C ABI of the MI355X (gfx950) implementation of the data-parallel hot
 * path of the Lazarus MoE layer (Lazarus: Resilient and Elastic Training of
 * Mixture-of-Experts Models, arXiv 2407.04656).
 *
 * One pass of the layer is five device calls on one stream
 *
 *     lz_route -> lz_plan_dispatch -> lz_permute (or lz_permute_scatter) -> lz_expert_ffn
 *              -> lz_unpermute_combine
 *
 * plus host-side planning (allocation, placement, re-planning after rank loss).  The N
 * logical ranks of a placement plan live in one GPU's memory; no call communicates.
 *
 * Conventions
 *   - Notation follows the paper: T tokens, d model dim, ffn hidden dim, E experts,
 *     top-k, N ranks, c replica slots per rank, S = N*c slots, P = T*k pairs; a "pair"
 *     is one (token t, choice kk) routing decision with pair index p = t*k + kk.
 *   - A plan is slot_expert[S], slot id s = rank*c + local slot: the paper's placement
 *     matrix (Appendix, proof of Theorem 1) read column by column.
 *   - Every function returns an int32 status: LZ_OK or a negative LZ_E* code; nothing
 *     throws.  lz_strerror() names a code.
 *   - "dev" pointers are device (HBM) addresses, "host" pointers are ordinary host
 *     memory.  The caller owns every buffer; the library allocates nothing and keeps no
 *     state between calls.  Scratch comes from a caller-provided device workspace whose
 *     size lz_*_workspace_bytes() reports.
 *   - Device calls are enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     default stream), return without waiting, and never synchronise with the host.
 *     Arguments that can be checked on the host are; data-dependent problems (an id out
 *     of range, an expert without a replica) are flagged in an optional device status
 *     word and never cause an out-of-bounds access.
 *   - All matrices are row-major and dense.  dtype LZ_BF16 tensors hold bfloat16 bit
 *     patterns; accumulation is always fp32.
 *   - Limits: 1 <= k <= min(E, 8), E <= 256, N <= 64, c <= 64, P = T*k <= 2^30 (buffers may exceed 4 GiB).
 */
#ifndef LAZARUS_MOE_H
#define LAZARUS_MOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum {
  LZ_OK = 0,
  LZ_EINVAL = -1,        /* null pointer / value out of the documented range          */
  LZ_ESHAPE = -2,        /* shape outside the limits above or not supported by a path  */
  LZ_EWORKSPACE = -3,    /* workspace missing, misaligned (256 B) or too small         */
  LZ_EUNRECOVERABLE = -4,/* an expert has no replica on any surviving rank (Sec. 4.3)  */
  LZ_EINFEASIBLE = -5,   /* fewer slots than experts                                   */
  LZ_EHIP = -6           /* a HIP runtime call failed (launch error)                   */
};

enum { LZ_F32 = 0, LZ_BF16 = 1 };
enum { LZ_GELU = 0, LZ_SWIGLU = 1 };

/* bits of the device status word written by lz_plan_dispatch */
enum {
  LZ_PLAN_UNCOVERED_EXPERT = 1,  /* an expert received tokens but the plan holds no replica */
  LZ_PLAN_BAD_EXPERT_ID = 2,     /* a top-k id or a slot_expert entry outside [0, E)        */
  LZ_PLAN_BAD_RANK_SPLIT = 4     /* rank_tok_off not ascending from 0 to T                  */
};

typedef struct {
  int32_t T, d, ffn, E, k, N, c;
  int32_t dtype; /* LZ_F32 | LZ_BF16: type of x, xp, hidden, yp, y and the weights */
  int32_t act;   /* LZ_GELU | LZ_SWIGLU */
} lz_shape;

const char* lz_strerror(int32_t code);
int32_t lz_version(void);

/* Bytes of device workspace (256-byte aligned) lz_plan_dispatch / lz_expert_ffn need
 * for this shape; 0 if the shape is invalid. */
size_t lz_plan_workspace_bytes(const lz_shape* shape);
size_t lz_ffn_workspace_bytes(const lz_shape* shape);

/* ---------------------------------------------------------------- device hot path */

/* Top-k gate routing (Sec. 2.1: the gate network routes each token to its top-k
 * experts).  For every token: the k largest of its E fp32 logits in descending order,
 * equal logits towards the lower expert index (-0.0 == +0.0); gates = softmax over
 * those k logits in fp32 (they sum to 1).  Logits must be finite.
 *   logits      dev [T,E] f32 (in)      topk_ids   dev [T,k] i32 (out)
 *   topk_gates  dev [T,k] f32 (out)
 * T == 0 is a no-op. */
int32_t lz_route(const float* logits, int32_t T, int32_t E, int32_t k,
                 int32_t* topk_ids, float* topk_gates, void* stream);

/* The flexible token dispatcher's schedule (Algorithm 1, Sec. 4.2) for all source ranks
 * at once, and the row maps of the per-slot contiguous buffers.
 *   1. Tej[e,i]: pairs routed to expert e whose token lies on rank i, rank i owning
 *      tokens [rank_tok_off[i], rank_tok_off[i+1])  (the algorithm's T_{e,j}; the
 *      all-gather of Sec. 4.2 is unnecessary in one address space).
 *   2. D[e,i,j]: pairs of e that rank i sends to rank j.  Integer reading of the
 *      algorithm: capacity cap[e,j] = floor(hi*t_e/r_e) - floor(lo*t_e/r_e) with lo/hi
 *      the running replica count before/after rank j; each rank keeps min(cap, Tej)
 *      (local tokens first); its overflow is spread over the other ranks in proportion
 *      to their residual capacity, cumulatively floored so every row of D sums to Tej.
 *   3. Row maps (the algorithm's reshuffle, extended to the receive side): rank i's
 *      pairs of e go, in token order, to destinations in ascending j; the (e,j) receive
 *      list is the concatenation over ascending i and is cut over the R[e,j] slots of
 *      rank j holding e (ascending slot id), slot m taking positions
 *      [floor(m*n/R), floor((m+1)*n/R)).  Rows are numbered slot after slot.
 * The result is deterministic (no order-dependent atomics).
 *   topk_ids     dev [T,k] i32 (in)       rank_tok_off dev [N+1] i32 (in)
 *   slot_expert  dev [S] i32 (in)
 *   slot_counts  dev [S] i32 (out)        slot_offsets dev [S+1] i32 (out, exclusive scan)
 *   pair_to_row  dev [P] i32 (out; -1 for a pair that could not be placed)
 *   row_to_pair  dev [P] i32 (out; inverse map, -1 for an unused row)
 *   Tej_opt      dev [E,N] i32 or NULL    D_opt dev [E,N,N] i32 or NULL (out, optional)
 *   status_opt   dev [1] i32 or NULL (out: 0 or LZ_PLAN_* bits)
 *   ws           dev workspace of >= lz_plan_workspace_bytes(shape) bytes */
int32_t lz_plan_dispatch(const int32_t* topk_ids, const lz_shape* shape,
                         const int32_t* rank_tok_off, const int32_t* slot_expert,
                         int32_t* slot_counts, int32_t* slot_offsets,
                         int32_t* pair_to_row, int32_t* row_to_pair,
                         int32_t* Tej_opt, int32_t* D_opt, int32_t* status_opt,
                         void* ws, size_t ws_bytes, void* stream);

/* lz_plan_dispatch for callers that cannot allocate or carry a workspace (code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc): same arguments minus the
 * workspace, same kernels, same results.  The tables live in a fixed array of
 * LZ_PLAN_NOALLOC_SCRATCH_BYTES of device memory inside the library (every GPU the library runs
 * on holds its own copy until the process ends; its address is looked up once per GPU, on the
 * first call there).  The call allocates nothing and frees nothing.
 * LZ_EWORKSPACE if lz_plan_workspace_bytes(shape) exceeds LZ_PLAN_NOALLOC_SCRATCH_BYTES (all five
 * benchmark configurations need less than 1 MiB).  All calls on one GPU share that GPU's array:
 * calls that overlap in time on one GPU (two streams, two threads) race; order them.  Nothing in
 * the array has to be cleared between calls. */
#define LZ_PLAN_NOALLOC_SCRATCH_BYTES (4u << 20)
int32_t lz_plan_dispatch_noalloc(const int32_t* topk_ids, const lz_shape* shape,
                                 const int32_t* rank_tok_off, const int32_t* slot_expert,
                                 int32_t* slot_counts, int32_t* slot_offsets,
                                 int32_t* pair_to_row, int32_t* row_to_pair,
                                 int32_t* Tej_opt, int32_t* D_opt, int32_t* status_opt,
                                 void* stream);

/* Reshuffle into per-slot contiguous buffers (Algorithm 1's h -> h'):
 * xp[row,:] = x[row_to_pair[row] / k, :]; rows whose map entry is outside [0,P) are
 * zero-filled.  x dev [T,d], xp dev [P,d], both of shape->dtype. */
int32_t lz_permute(const void* x, const int32_t* row_to_pair, const lz_shape* shape,
                   void* xp, void* stream);

/* The same reshuffle driven by the inverse map, token-major: xp[pair_to_row[t*k+kk], :] = x[t, :]
 * for every pair whose row lies in [0,P).  x is read once and written k times (the compulsory
 * traffic); rows of xp that no pair maps to are left untouched (they lie outside every slot
 * range, so lz_expert_ffn never reads them).  Same buffers and dtypes as lz_permute. */
int32_t lz_permute_scatter(const void* x, const int32_t* pair_to_row, const lz_shape* shape,
                           void* xp, void* stream);

/* One-time conversion between the usual [out, in] weight layout and the input-major layout the
 * FFN calls take (not on the timed path): packed[s][c][r] = w[s][r][c] for s < S, i.e.
 * w dev [S, rows, cols] -> packed dev [S, cols, rows], any sizes, dtype LZ_F32 or LZ_BF16.
 * w1 [S, n1, d] -> [S, d, n1] and w2 [S, d, ffn] -> [S, ffn, d]; applied to a gradient in the
 * library's layout it gives the [out, in] form back.  The buffers must not overlap. */
int32_t lz_pack_weights(const void* w, int32_t S, int32_t rows, int32_t cols, int32_t dtype, void* packed,
                        void* stream);

/* Expert FFN over the permuted buffer (Sec. 2.1: experts are parallel FFNs; each replica
 * processes the tokens dispatched to it).  Rows [slot_offsets[s], slot_offsets[s+1]) use
 * the weights of slot s:
 *   LZ_GELU    yp = gelu(xp W1) W2              gelu = 0.5 v (1 + erf(v/sqrt 2)), the erf form (not tanh);
 *                                                fp32 path: erff; bf16 MFMA path: erf to < 1e-6 absolute
 *   LZ_SWIGLU  yp = (silu(xp Wg) * (xp Wu)) W2
 *   w1  dev [S, d, n1]   n1 = ffn (GELU) or 2*ffn (SwiGLU: columns [0,ffn) = Wg, [ffn,2ffn) = Wu)
 *   w2  dev [S, ffn, d]
 * The weights are stored input-major (row = input feature, column = output feature, the
 * transpose of the usual [out, in] convention): the k-major tiles this gives the MFMA kernel
 * load in 512-byte runs and measured 2-4 % faster than [out, in].
 * Every slot owns its own copy of its expert's weights (replicas are separate buffers).
 * The hidden activation is kept in shape->dtype in the workspace; products accumulate
 * in fp32.  LZ_BF16 uses MFMA kernels when d % 256 == 0 and ffn % 128 == 0 (ffn % 256 for
 * GELU) and a generic tiled kernel otherwise; LZ_F32 always uses the generic kernel.
 * slot_offsets is read on the device only; offsets outside [0,P] are clipped.
 *   xp dev [P,d] (in), yp dev [P,d] (out, 16-byte aligned), ws >= lz_ffn_workspace_bytes(shape). */
int32_t lz_expert_ffn(const void* xp, const int32_t* slot_offsets,
                      const void* w1, const void* w2, const lz_shape* shape,
                      void* yp, void* ws, size_t ws_bytes, void* stream);

/* The three stages of lz_expert_ffn as separate calls, for callers that want to time or
 * interleave them; lz_expert_ffn is exactly tiles -> up -> down on the same workspace.
 *   lz_ffn_tiles  turns slot_offsets into the row-tile table and work queues kept in ws
 *   lz_ffn_up     hidden = act(xp W1) per slot, hidden kept in ws          (needs tiles)
 *   lz_ffn_down   yp = hidden W2 per slot                                  (needs up)
 * The MFMA GEMMs are persistent kernels that draw their tiles from queues in ws with atomic
 * tickets and reset the tickets when they finish, so up / down may be repeated on one table,
 * but a workspace serves one call at a time: calls on the same ws must be ordered (one
 * stream, or events), never concurrent. */
int32_t lz_ffn_tiles(const int32_t* slot_offsets, const lz_shape* shape, void* ws, size_t ws_bytes,
                     void* stream);
int32_t lz_ffn_up(const void* xp, const void* w1, const lz_shape* shape, void* ws, size_t ws_bytes,
                  void* stream);
int32_t lz_ffn_down(const void* w2, const lz_shape* shape, void* yp, void* ws, size_t ws_bytes,
                    void* stream);

/* The reshuffle fused into the first GEMM (Algorithm 1's h -> h' done by the consumer: the GEMM's
 * activation loads read x through the row map, so no permuted copy of x is written or read):
 *   lz_ffn_up_gather      hidden = act(x[row_to_pair[row] / k] W1) per slot   (replaces lz_permute + lz_ffn_up)
 *   lz_expert_ffn_gather  tiles -> up_gather -> down                           (replaces lz_permute + lz_expert_ffn)
 * Same results, bit for bit, as the unfused calls on the same inputs.  A row whose map entry is
 * outside [0,P) reads as zeros (no such row lies inside a slot).  x dev [T,d] of shape->dtype,
 * row_to_pair dev [P] i32 from lz_plan_dispatch; the other arguments as in lz_ffn_up / lz_expert_ffn.
 * The MFMA path addresses x with 32-bit byte offsets: LZ_ESHAPE if T*d*2 >= 2^32 there. */
int32_t lz_ffn_up_gather(const void* x, const int32_t* row_to_pair, const void* w1, const lz_shape* shape,
                         void* ws, size_t ws_bytes, void* stream);
int32_t lz_expert_ffn_gather(const void* x, const int32_t* row_to_pair, const int32_t* slot_offsets,
                             const void* w1, const void* w2, const lz_shape* shape,
                             void* yp, void* ws, size_t ws_bytes, void* stream);

/* Inverse permutation and gate-weighted combine (Sec. 2.1, the second all-to-all and the
 * combine): y[t,:] = sum_{kk<k} topk_gates[t,kk] * yp[pair_to_row[t*k+kk], :], summed in
 * fp32 in ascending kk and rounded once; a pair whose row is outside [0,P) contributes 0.
 *   yp dev [P,d], pair_to_row dev [P] i32, topk_gates dev [T,k] f32, y dev [T,d]. */
int32_t lz_unpermute_combine(const void* yp, const int32_t* pair_to_row,
                             const float* topk_gates, const lz_shape* shape,
                             void* y, void* stream);

/* ---------------------------------------------------------------- training: forward that keeps
 * its intermediates, and the backward pass.
 *
 * The paper trains the layer (Sec. 5: expert gradients are all-reduced over each expert's
 * replicas) without printing backward formulas; what these calls compute is the chain rule on
 * the forward of Sec. 2.1, one step per call, in reverse order:
 *
 *   lz_combine_backward   dgates[t,kk] = <dy[t], yp[row]>,  dyp[row] = gates[t,kk] dy[t]
 *   lz_ffn_backward       dH = dyp W2^T,  dW2[s] = H_s^T dyp_s,  dZ = dH * act'(Z),
 *                         dxp = dZ W1^T,  dW1[s] = xp_s^T dZ_s          (per slot s)
 *   lz_permute_backward   dx[t] = sum_kk dxp[row(t,kk)]
 *   lz_route_backward     dlogits[t, ids[t,j]] = g_j (dg_j - sum_i g_i dg_i), 0 elsewhere
 *   lz_reduce_replica_grads   dW[e] = sum of dW[s] over the slots s holding expert e
 *
 * Products are accumulated in fp32 and every stored tensor is rounded once to shape->dtype.
 * bf16 shapes with d % 256 == 0, ffn % 64 == 0, d*ffn*4 < 2^31 and N*c*max(d, 2*ffn) < 2^31 run on
 * the MFMA kernels, whatever the size of the activation tensors (tensor pointers 16-byte aligned there);
 * every other valid shape (fp32 tensors, other bf16 sizes) runs on plain tiled fp32-FMA kernels
 * that use erff / expf (the fp32 configuration meets its 1e-5 bar), as long as T*k/64 + N*c is
 * at most 65535.  All tensor pointers are device memory; `ws` is 256-byte aligned device memory of
 * lz_train_workspace_bytes(shape) bytes that serves one call at a time. */
size_t lz_train_workspace_bytes(const lz_shape* shape);

/* lz_expert_ffn that also returns what the backward needs: z = xp W1 (pre-activation,
 * [P, n1]; SwiGLU: columns [0,ffn) gate, [ffn,2ffn) up) and h = act(z) [P, ffn], both written
 * by the first GEMM's epilogue.  The activation is applied to the bf16-rounded z.  Rows outside
 * every slot are left untouched.
 *   xp dev [P,d], w1 dev [S,d,n1], w2 dev [S,ffn,d], z dev [P,n1] out, h dev [P,ffn] out, yp dev [P,d] out */
int32_t lz_ffn_forward_train(const void* xp, const int32_t* slot_offsets, const void* w1, const void* w2,
                             const lz_shape* shape, void* z, void* h, void* yp, void* ws, size_t ws_bytes,
                             void* stream);

/* Backward of lz_unpermute_combine.  A dyp row that no pair maps to is left untouched.
 *   dy dev [T,d], yp dev [P,d], dyp dev [P,d] out (all of shape->dtype), dgates dev [T,k] f32 out */
int32_t lz_combine_backward(const void* dy, const void* yp, const int32_t* pair_to_row,
                            const float* topk_gates, const lz_shape* shape, void* dyp, float* dgates,
                            void* stream);

/* Backward of the expert FFN over the permuted buffer.
 *   dyp, xp dev [P,d]; z dev [P,n1], h dev [P,ffn] from lz_ffn_forward_train
 *   w1 dev [S,d,n1], w2 dev [S,ffn,d]: the forward's weights, as they are
 *   dxp dev [P,d] out (rows outside every slot untouched)
 *   dw1 dev [S,d,n1] out, dw2 dev [S,ffn,d] out: each slot's own gradient in the weights' layout,
 *   zero for an empty slot */
int32_t lz_ffn_backward(const void* dyp, const void* xp, const void* z, const void* h,
                        const int32_t* slot_offsets, const void* w1, const void* w2,
                        const lz_shape* shape, void* dxp, void* dw1, void* dw2, void* ws,
                        size_t ws_bytes, void* stream);

/* lz_ffn_backward for training with micro-batches: the same computation, but each slot's weight
 * gradients are ADDED to fp32 accumulators instead of being stored (rounded) in the training dtype:
 *   dw1_acc dev [S,d,n1] f32, dw2_acc dev [S,ffn,d] f32 (in/out; the caller zeroes them before the
 *   first micro-batch; an empty slot adds nothing); 16-byte aligned.
 * lz_reduce_replica_grads_dtype(..., LZ_F32, ...) sums the accumulators over an expert's replicas. */
int32_t lz_ffn_backward_accumulate(const void* dyp, const void* xp, const void* z, const void* h,
                                   const int32_t* slot_offsets, const void* w1, const void* w2,
                                   const lz_shape* shape, void* dxp, float* dw1_acc, float* dw2_acc,
                                   void* ws, size_t ws_bytes, void* stream);

/* Backward of the reshuffle: dx[t,:] = sum_{kk<k} dxp[pair_to_row[t*k+kk], :], fp32 sum in
 * ascending kk, rounded once.  Same dtypes as lz_unpermute_combine.  dxp dev [P,d], dx dev [T,d] out. */
int32_t lz_permute_backward(const void* dxp, const int32_t* pair_to_row, const lz_shape* shape,
                            void* dx, void* stream);

/* Backward of the top-k softmax gates of lz_route (the selection is piecewise constant).
 *   dgates, topk_gates dev [T,k] f32; topk_ids dev [T,k] i32; dlogits dev [T,E] f32 out */
int32_t lz_route_backward(const float* dgates, const float* topk_gates, const int32_t* topk_ids,
                          const lz_shape* shape, float* dlogits, void* stream);

/* The sum an all-reduce over an expert's replica set leaves on every replica (Sec. 5), for
 * replicas that live on one device: dw[e] = sum over slots s with slot_expert[s] == e of
 * dw_slot[s], ascending s, fp32 sum, one rounding; an expert without a slot gets zero.
 *   dw_slot dev [S, elems_per_slot] bf16, slot_expert dev [S] i32, dw dev [E, elems_per_slot] bf16 out;
 *   elems_per_slot % 8 == 0, pointers 16-byte aligned
 * lz_reduce_replica_grads_dtype: the same for LZ_F32 or LZ_BF16 tensors of any size and alignment. */
int32_t lz_reduce_replica_grads(const void* dw_slot, const int32_t* slot_expert, int32_t S, int32_t E,
                                int64_t elems_per_slot, void* dw, void* stream);
int32_t lz_reduce_replica_grads_dtype(const void* dw_slot, const int32_t* slot_expert, int32_t S, int32_t E,
                                      int64_t elems_per_slot, int32_t dtype, void* dw, void* stream);

/* ---------------------------------------------------------------- host planning */

/* Replica allocation, Eq. 1 (Sec. 4.1): experts in ascending load t_e (ties: lower id)
 * get r_e = max(floor(t_e / sum_{e'>=e} t_e' * (N*c - sum_{e'<e} r_e')), f).  If the
 * remaining loads are all zero the remaining slots are split evenly; if N*c < E*f the
 * threshold is relaxed to floor(N*c/E).  Guarantees sum r_e = N*c, r_e >= f_eff and r_e
 * non-decreasing in load order.  All pointers host.  LZ_EINFEASIBLE if N*c < E. */
int32_t lz_allocate_replicas(const int64_t* t_e, int32_t E, int32_t N, int32_t c,
                             int32_t f, int32_t* r_e /* [E] out */);

/* Maximum-rank-overlap placement (Sec. 4.1; definition in Theorem 1).  Experts ordered by
 * (r_e, t_e, id) ascending are cut into ceil(E/c) groups of c; node group g takes the
 * next r_{first expert of g} ranks (the last group at most what is left) and each of its
 * ranks holds one replica of every expert of the group; if E <= c expert e also sits on
 * each of the first min(r_e,N) ranks.  Vacant slots, walked by (rank, local slot), take
 * the remaining replicas round-robin over the experts in that order.  sum r_e must equal
 * N*c and every r_e >= 1 (else LZ_EINVAL).  All pointers host. */
int32_t lz_place_mro(const int32_t* r_e, const int64_t* t_e, int32_t E, int32_t N,
                     int32_t c, int32_t* slot_expert /* [N*c] out */);

/* Spread baseline (Sec. 6.3): the q-th replica, listed expert after expert, goes to rank
 * q mod N, local slot q div N.  All pointers host. */
int32_t lz_place_spread(const int32_t* r_e, int32_t E, int32_t N, int32_t c,
                        int32_t* slot_expert /* [N*c] out */);

/* Compact baseline (Sec. 6.3): an expert's replicas on as few ranks as possible; replicas
 * listed expert after expert fill rank after rank (q-th replica: rank q div c, local slot
 * q mod c).  All pointers host. */
int32_t lz_place_compact(const int32_t* r_e, int32_t E, int32_t N, int32_t c,
                         int32_t* slot_expert /* [N*c] out */);

/* Probability that n_alive uniformly drawn alive ranks still hold every expert, by
 * enumerating all C(N, n_alive) sets (Sec. 6.3; the objective of Theorem 1).  Writes the
 * count of recoverable sets and the total.  N <= 62.  All pointers host. */
int32_t lz_recovery_probability(const int32_t* slot_expert, int32_t E, int32_t N, int32_t c,
                                int32_t n_alive, uint64_t* n_recoverable, uint64_t* n_total);

typedef struct {
  int32_t dst_slot; /* slot in the NEW plan (rank m = m-th surviving rank)            */
  int32_t src_slot; /* slot in the OLD plan whose weights are copied                  */
  int32_t expert;
  int32_t remote;   /* 1 if the source lies on another rank (a network fetch), else 0 */
} lz_transfer;

/* Re-plan after rank loss (Sec. 4.3).  survivors = ranks with alive[j] != 0, ascending.
 * LZ_EUNRECOVERABLE if some expert has no replica on a survivor.  Otherwise: Eq. 1 on
 * N_new*c_new slots, MRO placement, then the greedy node mapping (each physical survivor,
 * in ascending id, takes the unused plan node with the fewest experts it does not already
 * hold; lowest plan node on ties) and one transfer per new slot: from the rank's own
 * lowest old slot of that expert if it held one, else from a surviving owner, the
 * requests for one expert dealt round-robin over its owners in ascending rank, one fetch
 * per (rank, expert).
 *   old_slot_expert host [N_old*c_old]   alive host [N_old] (u8)   t_e host [E]
 *   new_slot_expert host [N_new*c_new] out      plan2phys host [N_new] out
 *   xfers host [*n_xfers capacity] out; *n_xfers in: capacity (>= N_new*c_new), out: count
 *   N_new_out host [1] out */
int32_t lz_replan(const int32_t* old_slot_expert, int32_t N_old, int32_t c_old,
                  const uint8_t* alive, const int64_t* t_e, int32_t E, int32_t c_new,
                  int32_t f, int32_t* new_slot_expert, int32_t* plan2phys,
                  lz_transfer* xfers, int32_t* n_xfers, int32_t* N_new_out);

/* Carry out a transfer list on the device: for each entry copy the source slot's w1 and
 * w2 blocks from the old weight buffers into the destination slot of the new ones
 * (device-to-device copies on `stream`; stands in for the batched send/recv of Sec. 5).
 *   xfers host [n]; w1_old/w2_old dev [S_old,...]; w1_new/w2_new dev [S_new,...]. */
int32_t lz_apply_transfers(const lz_transfer* xfers, int32_t n,
                           const void* w1_old, const void* w2_old, int32_t S_old,
                           void* w1_new, void* w2_new, int32_t S_new,
                           const lz_shape* shape, void* stream);

/* ---- diagnostics ------------------------------------------------------------------------- */

/* Records, for a launch shaped like the grouped GEMM's persistent kernel (256 threads and the
 * same LDS per workgroup, so one workgroup per CU), the id (0..7) of the XCD that each workgroup
 * ran on, read from the hardware's XCC_ID register.  The GEMM gives workgroup b the home queue
 * b % 8 on the expectation that consecutive workgroups go to consecutive XCDs; this call lets a
 * test or a user check that expectation on their machine (only cache locality depends on it).
 *   xcc_of_workgroup  dev [n_workgroups] i32 (out);  0 <= n_workgroups <= 65535 */
int32_t lz_debug_xcc_ids(int32_t* xcc_of_workgroup, int32_t n_workgroups, void* stream);

#ifdef __cplusplus
}
#endif
#endif /* LAZARUS_MOE_H */
