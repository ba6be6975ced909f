/*
 * feplb.h -- C ABI of the single-rank MoE hot path of FEPLB on MI355X (gfx950).
 *
 * One EP rank's expert computation after Two-Phase Dispatch (paper Section 2.2,
 * timeline in Section 2.3): route -> permute by static/dynamic expert group ->
 * ragged grouped SwiGLU expert FFN -> un-permute with weighted top-k combine,
 * plus the host-side greedy rebalancing plan and the staging copy of dynamic
 * experts' weights.
 *
 * Conventions shared by every entry point
 *   - returns FEPLB_OK (0) or a negative FEPLB_E* code; feplb_last_error() gives
 *     a thread-local text for the last failure on the calling thread;
 *   - arguments are validated on the host before anything is launched; a failed
 *     call launches nothing;
 *   - "device" pointers are HIP device memory of the current device, owned by the
 *     caller, 16-byte aligned; "host" pointers are ordinary host memory that may
 *     be released as soon as the call returns;
 *   - GPU work is enqueued on the caller's stream and never synchronises with
 *     the host; the library allocates and frees no device memory: scratch comes
 *     from the caller through the *_workspace_bytes() queries;
 *   - `stream`, `event` are hipStream_t / hipEvent_t passed as void*;
 *   - matrices are dense row-major; bf16 is the 16-bit brain float format;
 *   - the number of permuted rows R lives on the device (offsets[G]); calls that
 *     follow the permute take a capacity R_cap >= R for sizing.
 */
#ifndef FEPLB_H
#define FEPLB_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define FEPLB_OK 0
#define FEPLB_EINVAL (-1)     /* null pointer, negative size, unknown flag            */
#define FEPLB_ESHAPE (-2)     /* sizes outside what the kernels support              */
#define FEPLB_EALIGN (-3)     /* device pointer not 16-byte aligned                  */
#define FEPLB_EWORKSPACE (-4) /* workspace missing or too small                      */
#define FEPLB_EHIP (-5)       /* a HIP call failed; text in feplb_last_error()       */
#define FEPLB_ECAPACITY (-6)  /* output array (moves) too small                      */

#define FEPLB_F32 0
#define FEPLB_BF16 1

#define FEPLB_ORD_MAX 2147483647 /* open upper end of an ordinal window */

/* limits of this build */
#define FEPLB_MAX_EXPERTS 1024
#define FEPLB_MAX_TOPK 32
#define FEPLB_MAX_GROUPS 128

const char* feplb_version(void);
const char* feplb_last_error(void);

/* ------------------------------------------------------------------ routing
 * Section 2.3: every device first runs the router, whose per-token expert choices
 * drive everything that follows; the paper's model uses top-k routing over 128 routed experts with no auxiliary
 * loss (Section 3.1).  The paper does not give the score function; this build
 * uses softmax over all E logits, keeps the k largest and renormalises them to
 * sum to one.  Selection order: logit descending, expert id ascending on ties
 * (-0.0 equals +0.0); slot 0 holds the largest weight.
 *
 *   logits   device, fp32 [T,E], finite values (NaN/Inf: unspecified result)
 *   topk_ids device, int32 [T,k]   out
 *   topk_w   device, fp32  [T,k]   out, each row sums to 1
 *   counts   device, int32 [E]     out, assignments per expert; may be NULL
 * Limits: 1 <= k <= min(E, FEPLB_MAX_TOPK), E <= FEPLB_MAX_EXPERTS, T >= 0.
 */
int32_t feplb_route_topk(const float* logits, int32_t T, int32_t E, int32_t k,
                         int32_t* topk_ids, float* topk_w, int32_t* counts,
                         void* stream);

/* ------------------------------------------------------------------ permute
 * Section 2.2 Phase 1: tokens are "permuted" by expert on the device that will
 * run them; Section 2.3: a device's work splits into static experts and dynamic
 * (copied) experts.  A group is one expert's weight set applied to a window of
 * that expert's assignments: walking the flat assignments a = t*k + j in
 * ascending order, the i-th assignment to `expert` (i counted from 0) belongs
 * to the group when ord_lo <= i < ord_hi.  A static expert uses the window
 * [0, FEPLB_ORD_MAX); a replica that takes over part of an expert's batch uses
 * a sub-window.  Windows of one expert must not overlap.  Assignments that
 * match no group are not local and are dropped.
 *
 * Rows are laid out group after group in table order, ascending a inside a
 * group (stable), which makes every output unique.
 *
 *   topk_ids device, int32 [T,k]
 *   groups   host,   G entries
 *   X        device, bf16 [T,d]
 *   Xp       device, bf16 [R_cap,d]  out: Xp[r,:] = X[row_src[r] / k, :] for r < R
 *   offsets  device, int32 [G+1]     out: group g owns rows offsets[g]..offsets[g+1]-1; offsets[G] = R
 *   row_src  device, int32 [R_cap]   out: flat assignment of row r (entries >= R untouched)
 *   inv      device, int32 [T*k]     out: row of assignment a, or -1 when it is not local
 *   ws       device, feplb_permute_workspace_bytes(T,k,E,G) bytes of scratch
 * If R > R_cap, rows beyond R_cap are not written (offsets and inv still hold
 * the true values, so the caller can detect the overflow from offsets[G]).
 * Limits: d % 8 == 0, G <= FEPLB_MAX_GROUPS, E <= FEPLB_MAX_EXPERTS, T*k < 2^31.
 * With Xp NULL only the index arrays are computed (X is then ignored).
 */
typedef struct feplb_group {
  int32_t expert;
  int32_t ord_lo;
  int32_t ord_hi;
} feplb_group;

size_t feplb_permute_workspace_bytes(int32_t T, int32_t k, int32_t E, int32_t G);

int32_t feplb_permute(const int32_t* topk_ids, int32_t T, int32_t k, int32_t E,
                      const feplb_group* groups, int32_t G,
                      const void* X, int32_t d, void* Xp, int32_t R_cap,
                      int32_t* offsets, int32_t* row_src, int32_t* inv,
                      void* ws, size_t ws_bytes, void* stream);

/* Section 2.3, per-micro-batch timeline: the static experts' computation does not depend
 * on the rebalancing plan, so it can be permuted and started before the plan is known; the
 * dynamic experts' groups are added once it is.  feplb_permute_append takes the same
 * arguments as feplb_permute for those later groups and differs in three points:
 *   - offsets[0] is an INPUT read on the device: the row at which these groups start (the
 *     end of the earlier call, i.e. pass that call's `offsets + G_earlier`); offsets[1..G]
 *     are written as before;
 *   - inv entries of assignments that match none of THESE groups are left as they are, so the
 *     earlier call's rows survive (no assignment may match groups of both calls);
 *   - with X/Xp, only rows [offsets[0], offsets[G]) of Xp are written.
 * R_cap still bounds the highest row written.  Uses the same workspace size; the two calls may
 * share a workspace if they are ordered on the device.
 */
int32_t feplb_permute_append(const int32_t* topk_ids, int32_t T, int32_t k, int32_t E,
                             const feplb_group* groups, int32_t G,
                             const void* X, int32_t d, void* Xp, int32_t R_cap,
                             int32_t* offsets, int32_t* row_src, int32_t* inv,
                             void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------ expert FFN
 * Section 3.1: expert compute is a Grouped GEMM; Section 2.3: its efficiency
 * depends on each expert's batch size and per-expert launches fragment it
 * (Section 1).  One call runs a whole range of groups [g_begin, g_end) as a
 * single ragged launch per GEMM: for every row r of group g
 *     a = Xp[r,:] * W_gate[g]   b = Xp[r,:] * W_up[g]        (fp32 accumulate)
 *     H[r,:]  = bf16( a * sigmoid(a) * b )                    (phase GATE_UP)
 *     Yp[r,:] = H[r,:] * W_down[g]                            (phase DOWN)
 * The static range runs first; the dynamic range runs after the staging event
 * (Section 2.3 timeline), so a layer needs two calls, never one per expert.
 *
 *   Xp      device, bf16 [R_cap,d] -- or, with row_src, the unpermuted X [T,d]
 *   row_src device, int32 [R_cap] as written by feplb_permute (flat assignment
 *           indices t*k+j), or NULL.  When given, GATE_UP gathers its input rows
 *           while loading them: row r is X[row_src[r] / k, :], read from the matrix
 *           `Xp` points at, and no permuted copy of X is needed (call
 *           feplb_permute without X/Xp).  Token indices are clamped to [0, T);
 *           needs T*d*2 < 4 GiB.
 *   T, k    rows of X and assignments per token when row_src is given, ignored otherwise
 *   offsets device, int32 [G+1] as written by feplb_permute (read on the device)
 *   w_gate, w_up, w_down  host arrays of (g_end) device pointers indexed by g:
 *           W_gate[g], W_up[g] bf16 [d,f]; W_down[g] bf16 [f,d]; entries below
 *           g_begin are not read
 *   H       device, bf16 [R_cap,f]   written by GATE_UP, read by DOWN
 *   Yp      device, [R_cap,d] of yp_dtype (FEPLB_F32 or FEPLB_BF16), written by DOWN
 *   phases  any non-empty subset of FEPLB_FFN_SCHEDULE (turn offsets[] into the
 *           tile table kept in ws), FEPLB_FFN_GATE_UP, FEPLB_FFN_DOWN; the GEMM
 *           phases need a table built by an earlier or the same call with the
 *           same offsets, range and R_cap.  FEPLB_FFN_ALL does all three.
 *   ws      device, feplb_grouped_ffn_workspace_bytes(R_cap, G) bytes
 * Empty groups read no weights and do no work.
 * Limits: d % 256 == 0, f % 128 == 0, g_end <= FEPLB_MAX_GROUPS.
 */
#define FEPLB_FFN_GATE_UP 1
#define FEPLB_FFN_DOWN 2
#define FEPLB_FFN_SCHEDULE 4
#define FEPLB_FFN_ALL 7

size_t feplb_grouped_ffn_workspace_bytes(int32_t R_cap, int32_t G);

int32_t feplb_grouped_ffn(const void* Xp, const int32_t* row_src, int32_t T, int32_t k,
                          const int32_t* offsets,
                          int32_t g_begin, int32_t g_end, int32_t R_cap,
                          int32_t d, int32_t f,
                          const void* const* w_gate, const void* const* w_up,
                          const void* const* w_down,
                          void* H, void* Yp, int32_t yp_dtype, int32_t phases,
                          void* ws, size_t ws_bytes, void* stream);

/* The same call for callers that cannot allocate device memory or hand over a workspace: code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments,
 * results and limits as feplb_grouped_ffn, without ws / ws_bytes: the tile table lives in
 * FEPLB_STATIC_WS_BYTES of device memory that is part of the library itself (each GPU the library
 * runs on holds its own copy until the process ends).  Nothing is allocated or freed, by the
 * library or through any routine it calls.
 *   - Refused with FEPLB_ESHAPE when feplb_grouped_ffn_workspace_bytes(R_cap, g_end - g_begin)
 *     exceeds FEPLB_STATIC_WS_BYTES (256 KiB: about 4.1 million rows in 128 groups).
 *   - Every call on one GPU shares that GPU's table.  SCHEDULE rewrites the part it uses, so a
 *     later call with another range or fewer rows is safe; a GEMM phase without SCHEDULE runs on
 *     the table the last SCHEDULE on this GPU left.  Calls that overlap on one GPU (two streams,
 *     two threads) race on the table: order them.
 */
#define FEPLB_STATIC_WS_BYTES 262144

int32_t feplb_grouped_ffn_static(const void* Xp, const int32_t* row_src, int32_t T, int32_t k,
                                 const int32_t* offsets,
                                 int32_t g_begin, int32_t g_end, int32_t R_cap,
                                 int32_t d, int32_t f,
                                 const void* const* w_gate, const void* const* w_up,
                                 const void* const* w_down,
                                 void* H, void* Yp, int32_t yp_dtype, int32_t phases,
                                 void* stream);

/* ------------------------------------------------------------------ expert FFN, training
 * Section 3.2 reports the MoE layer's time per forward AND backward pass; the
 * backward of the Grouped GEMM of Section 3.1 is again grouped GEMMs over the same
 * ragged groups.  For every row r of group g, with a, b, H as above, s = sigmoid(a)
 * and the incoming gradient dYp[r,:]:
 *     dH = dYp[r,:] * W_down[g]^T
 *     da = dH * p,  p = b * s * (1 + a (1 - s))      db = dH * q,  q = a * s      (bf16)
 *     dXp[r,:] = da * W_gate[g]^T + db * W_up[g]^T
 *     dW_down[g] = sum_r H[r,:]^T dYp[r,:]   dW_gate[g] = sum_r Xp[r,:]^T da
 *     dW_up[g]   = sum_r Xp[r,:]^T db        (fp32, overwritten; zero for an empty group)
 *
 * feplb_grouped_ffn_train is feplb_grouped_ffn that also keeps what the backward
 * needs: AB, device bf16 [R_cap, 2f], receives the two partial derivatives of the
 * SwiGLU product, p = dH/da in columns [0,f) and q = dH/db in [f,2f), computed from
 * the fp32 products a, b while they are in registers (one rounding each).
 *
 * feplb_grouped_ffn_backward:
 *   Xp      device, bf16 [R_cap,d], the permuted rows (a materialised copy; no row_src here)
 *   offsets, g_begin, g_end, R_cap, d, f, w_gate, w_up, w_down   as in the forward call
 *   H       device, bf16 [R_cap,f]   as written by the forward call
 *   AB      device, bf16 [R_cap,2f]  in: p | q from feplb_grouped_ffn_train; out: da | db
 *   dYp     device, bf16 [R_cap,d]   gradient of the loss with respect to Yp
 *   dXp     device, [R_cap,d] of dxp_dtype (FEPLB_F32 or FEPLB_BF16)  out
 *   dw_gate, dw_up, dw_down  host arrays of (g_end) device pointers indexed by g:
 *           fp32 [d,f], [d,f], [f,d]  out
 *   WT      device scratch, feplb_grouped_ffn_backward_wt_bytes(g_end - g_begin, d, f)
 *           bytes: receives the transposed weights (phase TRANSPOSE), read by DGRAD
 *   phases  any non-empty subset of FEPLB_BWD_SCHEDULE (tile table from offsets[], as
 *           in the forward call; may be skipped when ws still holds the forward call's
 *           table for the same range), FEPLB_BWD_TRANSPOSE, FEPLB_BWD_DGRAD (needs
 *           the table and WT), FEPLB_BWD_WGRAD.  WGRAD for the gate and up matrices
 *           needs da | db, i.e. DGRAD in the same or an earlier call.  With
 *           FEPLB_BWD_ACCUMULATE added, WGRAD adds its results to what dw_gate, dw_up,
 *           dw_down hold (gradient accumulation over micro-batches; an empty group's
 *           matrices are then not touched) instead of overwriting them.
 *   ws      device, feplb_grouped_ffn_workspace_bytes(R_cap, g_end - g_begin) bytes
 * Rows past offsets[g_end] are neither read into any result nor written.
 * Limits: d % 256 == 0, f % 256 == 0, g_end <= FEPLB_MAX_GROUPS, R_cap >= 32 for WGRAD.
 */
#define FEPLB_BWD_SCHEDULE 1
#define FEPLB_BWD_TRANSPOSE 2
#define FEPLB_BWD_DGRAD 4
#define FEPLB_BWD_WGRAD 8
#define FEPLB_BWD_ALL 15
#define FEPLB_BWD_ACCUMULATE 16

int32_t feplb_grouped_ffn_train(const void* Xp, const int32_t* row_src, int32_t T, int32_t k,
                                const int32_t* offsets,
                                int32_t g_begin, int32_t g_end, int32_t R_cap,
                                int32_t d, int32_t f,
                                const void* const* w_gate, const void* const* w_up,
                                const void* const* w_down,
                                void* H, void* AB, void* Yp, int32_t yp_dtype, int32_t phases,
                                void* ws, size_t ws_bytes, void* stream);

size_t feplb_grouped_ffn_backward_wt_bytes(int32_t n_groups, int32_t d, int32_t f);

int32_t feplb_grouped_ffn_backward(const void* Xp, const int32_t* offsets,
                                   int32_t g_begin, int32_t g_end, int32_t R_cap,
                                   int32_t d, int32_t f,
                                   const void* const* w_gate, const void* const* w_up,
                                   const void* const* w_down,
                                   const void* H, void* AB, const void* dYp,
                                   void* dXp, int32_t dxp_dtype,
                                   void* const* dw_gate, void* const* dw_up, void* const* dw_down,
                                   void* WT, size_t wt_bytes, int32_t phases,
                                   void* ws, size_t ws_bytes, void* stream);

/* ------------------------------------------------------------------ combine
 * Section 2.3: the last step of a micro-batch hands the experts' outputs back to the
 * tokens' source devices (Combine); this is its local part: Y[t,:] = sum over slots j with inv[t*k+j] >= 0 of
 * topk_w[t,j] * Yp[inv[t*k+j],:], summed in fp32 in ascending j and rounded
 * once to bf16.  Tokens with no local slot get +0.
 *
 *   Yp device [R_cap,d] of yp_dtype; inv device int32 [T*k]; topk_w device fp32 [T,k]
 *   R_cap rows that Yp holds.  feplb_permute keeps the true row numbers in inv when the
 *         permutation overflowed its capacity; a slot whose row is >= R_cap was never
 *         computed, is treated as not local and is never read.
 *   Y  device, bf16 [T,d]  out
 * Limits: d % 8 == 0, k <= FEPLB_MAX_TOPK.
 */
int32_t feplb_unpermute_combine(const void* Yp, int32_t yp_dtype, int32_t R_cap,
                                const int32_t* inv, const float* topk_w,
                                int32_t T, int32_t k, int32_t d, void* Y,
                                void* stream);

/* ------------------------------------------------------------------ combine and router, backward
 * Section 3.2 times the layer's backward pass; these are the gradients of its
 * memory-bound steps (the grouped FFN's are above).  With dY[t,:] the gradient of the
 * loss with respect to Y:
 *     dYp[inv[t*k+j],:] = bf16( topk_w[t,j] * dY[t,:] )       for every local slot
 *     dw[t,j] = sum_i dY[t,i] * Yp[inv[t*k+j],i]  (fp32)      0 for a slot that is not local
 * and, the routing weights being the softmax of the k kept logits,
 *     dlogits[t, topk_ids[t,j]] = w_j (dw_j - sum_i w_i dw_i)  0 for every expert not kept.
 * The gradient of the row gather, dX[t,:] = sum over local slots of dXp[inv[t*k+j],:], is
 * feplb_unpermute_combine(dXp, inv, unit weights).
 *
 *   dY      device, bf16 [T,d]
 *   Yp      device, [R_cap,d] of yp_dtype, the expert outputs of the forward pass
 *   R_cap   rows of Yp and dYp; a slot whose row in inv is >= R_cap counts as not local
 *           (nothing is read or written for it, its dw is 0)
 *   dYp     device, bf16 [R_cap,d]  out (rows no slot refers to are left alone)
 *   dw      device, fp32 [T,k]      out
 *   dlogits device, fp32 [T,E]      out
 * Limits: d % 8 == 0, k <= FEPLB_MAX_TOPK, E <= FEPLB_MAX_EXPERTS.
 */
int32_t feplb_combine_backward(const void* dY, const void* Yp, int32_t yp_dtype, int32_t R_cap,
                               const int32_t* inv, const float* topk_w,
                               int32_t T, int32_t k, int32_t d, void* dYp, float* dw,
                               void* stream);
int32_t feplb_route_topk_backward(const int32_t* topk_ids, const float* topk_w, const float* dw,
                                  int32_t T, int32_t E, int32_t k, float* dlogits, void* stream);

/* ------------------------------------------------------------------ staging
 * Section 2.2 Phase 2 / Section 2.3: a dynamic expert's weights are copied into
 * a buffer of max_num_dyn x W_expert slots by a copy engine, off the compute
 * units, while the static experts run.  This enqueues hipMemcpyAsync(slot, src,
 * bytes) on `side_stream` and, if `done` is not NULL, records it there; the
 * compute stream then waits with feplb_stream_wait.  src may be device memory
 * or pinned host memory.
 */
int32_t feplb_stage_weights(void* slot, const void* src, size_t bytes,
                            void* side_stream, void* done_event);
int32_t feplb_stream_wait(void* stream, void* event);

/* size in bytes of one expert's gate, up and down matrices (Section 2.3: W_expert) */
size_t feplb_expert_bytes(int32_t d, int32_t f, int32_t elem_bytes);

/* ------------------------------------------------------------------ plan (host only, no HIP)
 * Section 2.3, load balancer: given the per-expert token counts every device
 * knows after Phase 1 (Section 2.2), decide which dynamic experts to copy where.
 *
 * FEPLB_PLAN_WHOLE is the paper's greedy: repeat { src = most loaded rank;
 * dst = least loaded other rank with a free slot; among src's own dynamic
 * experts that have not moved and hold >= max(tau,1) rows, busiest first, take
 * the first whose whole batch leaves dst strictly below src's load; move it }
 * until no such expert or receiver exists.  Ties go to the lowest id.  Whole
 * experts only, deterministic, so every rank derives the same plan.
 *
 * FEPLB_PLAN_OVERFLOW is not in the paper: it replicates on `this_rank` the
 * slots[this_rank] busiest dynamic experts owned elsewhere and hands it the
 * LAST rows_i occurrences of each (ord_lo = n - rows_i), sized so this_rank
 * ends at most at the balanced mean ceil(sum n / P).  this_rank < 0 picks the
 * rank whose own load is closest to half that mean and reports it in
 * *chosen_rank.
 *
 *   P ranks, E experts; owner[E] in [0,P); n[E] >= 0 rows per expert;
 *   dyn_flag[E] nonzero = eligible for copying; slots[P] >= 0 free buffer slots;
 *   moves[max_moves] out; *n_moves out; load_before[P], load_after[P] out (may be NULL);
 *   chosen_rank out (may be NULL).
 * All pointers are host memory.
 */
#define FEPLB_PLAN_WHOLE 0
#define FEPLB_PLAN_OVERFLOW 1

typedef struct feplb_move {
  int32_t expert;
  int32_t src;
  int32_t dst;
  int32_t reserved;
  int64_t rows;    /* rows that run on dst                       */
  int64_t ord_lo;  /* first ordinal of the window that dst takes */
} feplb_move;

int32_t feplb_plan(int32_t P, int32_t E, const int32_t* owner, const int64_t* n,
                   const uint8_t* dyn_flag, const int32_t* slots, int64_t tau,
                   int32_t mode, int32_t this_rank,
                   feplb_move* moves, int32_t max_moves, int32_t* n_moves,
                   int64_t* load_before, int64_t* load_after,
                   int32_t* chosen_rank);

/* ------------------------------------------------------------------ macro level: placement from history (host only)
 * Section 2.3 (and the system figure): beside the per-micro-batch balancer, a Router Predictor
 * re-assigns experts to devices now and then from routing history, at checkpoint time so that
 * the migration cost is spread out.  The paper gives no algorithm; this build's rule:
 *
 * feplb_history_update keeps an exponential moving average of the per-expert counts in fixed
 * point (FEPLB_HIST_FRAC_BITS fractional bits, so every rank derives the same integers):
 *     hist[e] += floor(((n[e] << 16) - hist[e]) / 2^shift)     decay 1 - 2^-shift per call
 * (shift = 0 keeps the last batch only).  0 <= shift <= 30, 0 <= n[e] < 2^46.
 *
 * feplb_place derives a new expert -> rank map: longest processing time first -- experts by
 * history, largest first (lowest id on ties), each to the bin with the least accumulated
 * history among the bins that hold fewer than `cap` experts (lowest bin on ties).  The new map
 * is taken only if its largest bin is strictly below the largest rank load of owner_in under
 * the same history (otherwise owner_out = owner_in and *n_migrated = 0).  Bins are named after
 * ranks so that many experts stay: the (bin, rank) pair sharing the most experts first (lowest
 * bin, then lowest rank on ties).  Needs cap * P >= E.  load_before / load_after [P] are the
 * predicted rank loads under owner_in / owner_out (may be NULL); *n_migrated counts experts
 * whose rank changes (may be NULL).
 *
 * feplb_mark_dynamic flags on every rank its `dyn` experts with the largest history (lowest id
 * on ties) as the dynamic ones (Section 2.3 gives only their number).
 * All pointers are host memory.
 */
#define FEPLB_HIST_FRAC_BITS 16

int32_t feplb_history_update(int32_t E, int64_t* hist, const int64_t* n, int32_t shift);
int32_t feplb_place(int32_t P, int32_t E, const int64_t* hist, int32_t cap, const int32_t* owner_in,
                    int32_t* owner_out, int64_t* load_before, int64_t* load_after,
                    int32_t* n_migrated);
int32_t feplb_mark_dynamic(int32_t P, int32_t E, const int32_t* owner, const int64_t* hist,
                           int32_t dyn, uint8_t* dyn_flag);

/* ------------------------------------------------------------------ straggler bookkeeping (host only)
 * Section 3.1, Metrics: the straggler of a per-rank quantity (tokens, or grouped-GEMM time) is
 * its maximum over the ranks minus its mean.  feplb_apply_moves gives the rank on which each
 * expert runs once a plan's whole-expert moves are applied (home[e] = owner[e] unless a move
 * names e, then its dst).
 */
int32_t feplb_apply_moves(int32_t P, int32_t E, const int32_t* owner, const feplb_move* moves,
                          int32_t n_moves, int32_t* home);
int32_t feplb_straggler(int32_t P, const double* per_rank, double* straggler);

#ifdef __cplusplus
}
#endif
#endif /* FEPLB_H */
