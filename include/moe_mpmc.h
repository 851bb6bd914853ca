/*
 * moe_mpmc.h -- C ABI of the MI355X (gfx950) library for the Switch-style top-1 MoE layer
 * forward with predictor-driven dynamic expert replication.
 *
 * The calls follow the data flow of the paper's two algorithms: the hash-building thread
 * (Algorithm 2) predicts an expert id per token (sru_predict); the inference thread
 * (Algorithm 1) turns the predicted ids into per-expert replica counts within a cap
 * (replica_plan), re-points tokens to physical replicas (moe_dispatch) and runs the
 * specialised model (moe_route for the gate, moe_expert_ffn, moe_combine).
 *
 * Conventions (all calls)
 *  - Every tensor pointer is a DEVICE pointer owned by the caller, row-major, contiguous,
 *    16-byte aligned.  The library never allocates, frees or keeps device memory; scratch
 *    space is a caller-supplied workspace whose size the *_workspace_bytes functions give.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls enqueue
 *    kernels and return without synchronising.  Data-dependent sizes (rows kept, slot
 *    ranges) stay in device memory; grids are sized for the worst case.
 *  - dtype: MOE_F32 = binary32 tensors; MOE_BF16 = bfloat16 tensors, products accumulated
 *    in binary32.  Index tensors are int32, probabilities binary32.
 *  - Return value: MOE_OK or a negative error code.  Arguments are validated on the host
 *    before anything is launched; on error nothing has been enqueued (MOE_ERR_HIP excepted).
 *    moe_last_error() returns a thread-local message for the last failing call.
 *  - Empty batches (T = 0, B = 0, max_rows = 0) are valid: sizes and flags are still checked,
 *    data pointers are not looked at and may be NULL; moe_route, sru_predict, moe_expert_ffn and
 *    moe_combine then enqueue nothing, replica_plan, moe_dispatch and moe_plan_dispatch write
 *    the tables of a batch without tokens (every expert one empty slot).
 *  - No C++ exception crosses the boundary.  Calls on different streams may overlap only if
 *    they use different workspaces and outputs.
 */
#ifndef MOE_MPMC_H
#define MOE_MPMC_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define MOE_OK 0
#define MOE_ERR_INVALID_ARG (-1) /* null pointer, negative size, misaligned shape          */
#define MOE_ERR_UNSUPPORTED (-2) /* dtype / shape / layout outside the built kernels       */
#define MOE_ERR_WORKSPACE (-3)   /* workspace missing or smaller than *_workspace_bytes    */
#define MOE_ERR_HIP (-4)         /* the HIP runtime refused a launch                       */

#define MOE_F32 0
#define MOE_BF16 1

#define MOE_MAX_EXPERTS 1024 /* E  <= 1024 */
#define MOE_MAX_TOPK 8       /* k  <= 8 (top-k routing) */
#define MOE_MAX_SLOTS 4096   /* E + replica budget <= 4096 */

#define MOE_LAYOUT_PLAIN 0  /* [E, K, N] row-major                                        */
#define MOE_LAYOUT_PACKED 1 /* image written by moe_pack_weights                          */

#define MOE_SCHEDULE_SLOTS 0   /* one stream of row tiles per physical slot (replication on) */
#define MOE_SCHEDULE_EXPERTS 1 /* one work item per logical expert walks all its rows        */

const char *moe_last_error(void);
int moe_version(void);
/* Identifier of the sources this binary was compiled from (a hash the build step passes in; "unknown"
 * for a build made some other way).  The Python binding compares it with the sources beside it. */
const char *moe_build_id(void);

/* ---------------------------------------------------------------------------------------
 * moe_route -- the softmax gate of the top-1 layer (Methodology: the model run is a
 * Switch-Transformer-like top-1 layer; Preliminaries: routing via softmax).
 *   logit[s][e] = sum_k x[s][k] * w_router[k][e] + b_router[e]
 *   expert_idx[s]  = argmax_e logit[s][e]          (lowest e on an exact tie)
 *   expert_prob[s] = softmax(logit[s])[expert_idx[s]]
 * x [T,d]; w_router [d,E]; b_router [E] binary32 or NULL (= 0); logits_opt [T,E] binary32
 * or NULL.  Sums, exponentials and the argmax are taken in binary32 for both dtypes.
 * w_layout: MOE_LAYOUT_PLAIN = row-major [d,E] (re-laid into the workspace on every call), or
 * MOE_LAYOUT_PACKED = the image moe_pack_weights writes for a [1,d,E] tensor (static router
 * weights packed once; bf16 with E = 128 or 256 and d a multiple of 128 only).
 * d must be a multiple of 8.  T = 0 is a no-op.
 */
size_t moe_route_workspace_bytes(int T, int d, int E, int dtype);
int moe_route(const void *x, const void *w_router, int w_layout, const float *b_router, int T, int d,
              int E, int dtype, int32_t *expert_idx, float *expert_prob, float *logits_opt, void *ws,
              size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------
 * Top-k routing (Experiments, setup: one of the two tasks is run with top-3 routing).  The paper
 * names the setting only; the reading built here is the usual one for a softmax gate:
 *   choice j = 0..k-1 of token s: the expert with the j-th largest logit (lower id first among
 *   equal logits); its weight is softmax(logit[s])[e_j], divided by the sum of the k weights when
 *   renormalize = 1;  an assignment is numbered a = j*T + s (all first choices before all second
 *   choices, which is also their priority under the capacity limit).
 * moe_route_topk: expert_idx and expert_weight hold k*T entries in that order (entry j*T + s);
 *   k = 1 gives moe_route's results bit for bit.  1 <= k <= min(MOE_MAX_TOPK, E).  Everything
 *   else as moe_route (same workspace size).
 * replica_plan takes the k*T ids as its batch.
 * moe_dispatch_topk: moe_dispatch over the k*T assignments (expert_idx, perm, inv hold k*T
 *   entries; workspace of moe_dispatch_workspace_bytes(k*T, E)); x still has T rows:
 *   x_perm[inv[a]] = x[a mod T], and row_token[r] = perm[r] mod T for r < K, -1 for K <= r < k*T
 *   (the row table moe_expert_ffn_rows gathers through).  x and x_perm may both be NULL.
 * moe_expert_ffn_rows: moe_expert_ffn with a gather (row_index required) from a matrix of
 *   n_x_rows rows, which need not equal max_rows; an index outside [0, n_x_rows) is never
 *   dereferenced.  Workspace as moe_expert_ffn.
 * moe_combine_topk: inv and expert_weight hold k*T entries;
 *   out[s] = (residual ? x[s] : 0) + sum over j with inv[j*T+s] >= 0, in the order j = 0..k-1, of
 *            expert_weight[j*T+s] * y_perm[inv[j*T+s]]   (binary32 multiply-adds, rounded once);
 *   a token with no kept choice: out[s] = x[s] bit for bit.  k = 1 is moe_combine.
 */
int moe_route_topk(const void *x, const void *w_router, int w_layout, const float *b_router, int T,
                   int d, int E, int dtype, int k, int renormalize, int32_t *expert_idx,
                   float *expert_weight, float *logits_opt, void *ws, size_t ws_bytes, void *stream);
int moe_dispatch_topk(const void *x, const int32_t *expert_idx, const int32_t *replicas, int T, int k,
                      int d, int E, int slot_capacity, int max_slots, int dtype, int32_t *counts,
                      int32_t *kept, int32_t *expert_offset, int32_t *slot_offset, int32_t *perm,
                      int32_t *inv, int32_t *row_token, void *x_perm, void *ws, size_t ws_bytes,
                      void *stream);
int moe_expert_ffn_rows(const void *x, int n_x_rows, const int32_t *row_index, const void *w1,
                        const void *w2, int weight_layout, const int32_t *slot_offset,
                        const int32_t *slot_expert, const int32_t *n_slots, int max_rows, int max_slots,
                        int E, int d, int F, int dtype, int schedule, void *y_perm, void *ws,
                        size_t ws_bytes, void *stream);
int moe_combine_topk(const void *y_perm, const void *x, const int32_t *inv, const float *expert_weight,
                     int T, int k, int d, int dtype, int residual, void *out, void *stream);

/* ---------------------------------------------------------------------------------------
 * sru_predict -- the expert predictor h_l of Algorithm 2 (the step that assigns a token its expert): a stack
 * of SRU layers (equations of the subsection "Simple Recurrent Unit (SRU) for expert
 * prediction") followed by a linear head and an argmax.
 *   per layer and sequence, t = 0..L-1, c_{-1} = 0:
 *     x' = W x_t;  f = sigmoid(W_f x_t + b_f);  r = sigmoid(W_r x_t + b_r)
 *     c_t = f*c_{t-1} + (1-f)*x';   h_t = r*tanh(c_t) + (1-r)*hw_t
 *     hw_t = x_t when the layer's input width equals n_hidden, else W_h x_t
 *   logits = h_last W_head + b_head;  pred_idx = argmax (lowest index on a tie)
 * The struct and every array it points to live in HOST memory; the weight tensors they name
 * are device pointers.  w_cat[l] is [n_in_l, k_l*n_hidden], column blocks W | W_f | W_r and,
 * when n_in_l != n_hidden (k_l = 4), W_h; n_in_0 = n_in, n_in_l = n_hidden afterwards.
 * b_f / b_r: arrays of n_layers device pointers to [n_hidden] binary32, or NULL (all zero);
 * single entries may be NULL too.  w_head [n_hidden, n_out]; b_head [n_out] or NULL.
 * emb [B, L, n_in].  Only MOE_BF16 is built; n_in a multiple of 64, n_hidden a multiple of
 * 128, n_out a multiple of 8 and <= MOE_MAX_EXPERTS.  Layer outputs are stored as bfloat16
 * between layers.
 */
typedef struct sru_weights {
    int n_layers, n_in, n_hidden, n_out;
    int w_layout; /* MOE_LAYOUT_PLAIN, or MOE_LAYOUT_PACKED: every w_cat[l] and w_head is the image
                     moe_pack_weights writes for it as a [1, K, N] tensor (n_out = 128 or 256 only) */
    const void *const *w_cat;
    const float *const *b_f;
    const float *const *b_r;
    const void *w_head;
    const float *b_head;
    int attention; /* 0: the head reads the last layer's states h_t.  1: sparsemax self-attention first
                      (the predictor's sparse attention: Methodology; SRU subsection, last paragraph --
                      the paper prints no equations, this is the reading built): inside
                      each sequence s[t,j] = <h_t,h_j>/sqrt(n_hidden), a[t,:] = sparsemax(s[t,:]) (the
                      Euclidean projection onto the simplex: exact zeros for less relevant positions),
                      z_t = h_t + sum_j a[t,j] h_j rounded to dtype, and the head reads z_t.
                      Needs L <= 1024 and n_hidden <= 256. */
} sru_weights;

size_t sru_predict_workspace_bytes(const sru_weights *w, int B, int L, int dtype);
int sru_predict(const void *emb, const sru_weights *w, int B, int L, int dtype, int32_t *pred_idx,
                float *logits_opt /* [B*L, n_out] or NULL */, void *ws, size_t ws_bytes,
                void *stream);

/* ---------------------------------------------------------------------------------------
 * replica_plan -- Algorithm 1's replication pass under the cap of the subsection "Capacity
 * capping".  From the ids idx[T] (predicted, or the router's own):
 *   n_e = #{s : idx[s] = e};  every expert owns one slot;
 *   want_e = max(0, ceil(n_e / slot_capacity) - 1) further replicas (slot_capacity = 1 is the
 *   algorithm as printed: one replica per further token);  D = sum want_e;
 *   D <= budget : replicas[e] = 1 + want_e;
 *   otherwise the budget is divided by the number of replicas still to be added:
 *     policy 0: replicas[e] = 1 + floor(budget*want_e / D), and the slots the floors leave
 *               go one by one to the expert with the largest n_e / replicas[e] among those
 *               still below 1 + want_e (lowest id on a tie);
 *     policy 1: equal shares among the experts that still want replicas, repeated until the
 *               share is 0, the remainder as in policy 0.
 * Outputs: plan_counts[E] = n_e; replicas[E]; slot_base[E+1] = exclusive scan of replicas;
 * slot_expert[E+budget] (slot -> expert, expert-major; unused tail = -1); n_slots[1].
 * Integer-only; ids outside [0,E) are ignored.  E <= MOE_MAX_EXPERTS, E+budget <=
 * MOE_MAX_SLOTS.
 */
size_t replica_plan_workspace_bytes(int T, int E); /* 0 for small batches: ws may then be NULL */
int replica_plan(const int32_t *idx, int T, int E, int budget, int slot_capacity, int policy,
                 int32_t *plan_counts, int32_t *replicas, int32_t *slot_base,
                 int32_t *slot_expert, int32_t *n_slots, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------
 * moe_dispatch -- capacity-limited dispatch of tokens to physical slots (Algorithm 1: a token
 * is re-pointed to a replica index; the inference-thread subsection: tokens are processed in
 * parallel while the batch stays within the capacity of the experts on the GPU).
 *   counts[e] = n_e (actual ids);  kept[e] = min(n_e, replicas[e]*slot_capacity);
 *   expert_offset[E+1] = exclusive scan of kept;  K = expert_offset[E];
 *   j(s) = rank of s among earlier tokens of its expert; kept iff j(s) < replicas[e]*C;
 *   inv[s] = expert_offset[e] + j(s) or -1;  perm[inv[s]] = s;  perm[K..T) = -1;
 *   x_perm[inv[s]] = x[s];  rows K..T of x_perm are left untouched;
 *   slot k of expert e covers q + (k < rem) consecutive rows (q, rem = kept[e] div/mod
 *   replicas[e]); slot_offset[max_slots+1] holds the first row of every slot, expert-major,
 *   entries from sum(replicas) on hold K.
 * replicas may be NULL (one slot per expert).  d*sizeof(element) must be a multiple of 16.
 * Ids must lie in [0,E).  Deterministic: no result depends on atomics order.
 */
size_t moe_dispatch_workspace_bytes(int T, int E);
int moe_dispatch(const void *x, const int32_t *expert_idx, const int32_t *replicas, int T, int d,
                 int E, int slot_capacity, int max_slots, int dtype, int32_t *counts,
                 int32_t *kept, int32_t *expert_offset, int32_t *slot_offset, int32_t *perm,
                 int32_t *inv, void *x_perm, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------
 * moe_dispatch_static -- moe_dispatch for callers that cannot allocate device memory (code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): same arguments, outputs
 * and kernels, but the per-block histograms live in a static device array of the library (1 MiB on
 * every GPU the library runs on, held until the process ends) instead of a caller's workspace.
 * Limit: ceil(T/1024) * E <= 262144 table entries (e.g. T <= 1048576 at E = 256); beyond it
 * MOE_ERR_UNSUPPORTED.  The call allocates and frees nothing; the first call on a device asks the
 * runtime for the array's address on that device (make one call outside any graph capture first).
 * Nothing in the array has to be cleared between calls (every entry read was written by the same
 * call).  All calls on one GPU share that GPU's array: calls that overlap on one GPU (different
 * streams, or different host threads without ordering) race; order them or use moe_dispatch.
 */
int moe_dispatch_static(const void *x, const int32_t *expert_idx, const int32_t *replicas, int T, int d,
                        int E, int slot_capacity, int max_slots, int dtype, int32_t *counts,
                        int32_t *kept, int32_t *expert_offset, int32_t *slot_offset, int32_t *perm,
                        int32_t *inv, void *x_perm, void *stream);

/* ---------------------------------------------------------------------------------------
 * moe_plan_dispatch -- replica_plan (Algorithm 1 with the budget cap) on plan_idx[n_plan], then the
 * index tables of moe_dispatch (moe_dispatch_topk for k > 1) for expert_idx[k*T] under that plan, as
 * one call: the same tables, bit for bit, as the two calls with max_slots = E + budget and no row
 * copy.  Small batches (n_plan and k*T at most 8192, E at most 256) run in a single kernel and need no
 * workspace; larger ones run the separate kernels.  row_token may be NULL when k = 1.
 */
size_t moe_plan_dispatch_workspace_bytes(int n_plan, int T, int k, int E);
int moe_plan_dispatch(const int32_t *plan_idx, int n_plan, const int32_t *expert_idx, int T, int k,
                      int E, int budget, int slot_capacity, int policy, int32_t *plan_counts,
                      int32_t *replicas, int32_t *slot_base, int32_t *slot_expert, int32_t *n_slots,
                      int32_t *counts, int32_t *kept, int32_t *expert_offset, int32_t *slot_offset,
                      int32_t *perm, int32_t *inv, int32_t *row_token, void *ws, size_t ws_bytes,
                      void *stream);

/* ---------------------------------------------------------------------------------------
 * moe_pack_weights -- one-time re-layout of static expert weights for the bf16 matrix-core
 * kernels (inference weights do not change between batches).  Input w [E, K, N] row-major
 * bf16, K a multiple of 8, N a multiple of 32.  Output, in 16-byte pieces of 8 consecutive k:
 * piece ((e*(N/32) + n/32)*(K/8) + k/8)*32 + n%32 holds w[e][8*(k/8) .. 8*(k/8)+7][n], i.e.
 * columns are grouped in strips of 32 and a strip is stored front to back along k, so a
 * wavefront that owns a strip streams it from HBM in address order.
 * moe_packed_weights_bytes gives the output size (equal to the input size).
 */
size_t moe_packed_weights_bytes(int E, int K, int N, int dtype);
int moe_pack_weights(const void *w, int E, int K, int N, int dtype, void *w_packed, void *stream);

/* ---------------------------------------------------------------------------------------
 * moe_expert_ffn -- the experts and their replicas process their tokens concurrently
 * (Abstract; contribution 2).  For every slot p < n_slots[0], e = slot_expert[p], rows
 * slot_offset[p] .. slot_offset[p+1]-1 of x_perm:
 *   h = relu(x_perm[row] W1[e])  (stored in dtype),   y_perm[row] = h W2[e]  (stored in dtype)
 * W1 [E,d,F], W2 [E,F,d].  MOE_F32 takes MOE_LAYOUT_PLAIN; MOE_BF16 takes MOE_LAYOUT_PACKED
 * (each of W1, W2 packed with moe_pack_weights, K = d resp. F) and needs d % 128 == 0,
 * F % 128 == 0.  schedule: MOE_SCHEDULE_SLOTS gives every slot its own row tiles, so the
 * replicas of a hot expert run side by side; MOE_SCHEDULE_EXPERTS makes one work item per
 * (expert, column tile) walk all rows of that expert one tile after another (tokens queue on
 * the one physical expert).  Both produce the same y_perm.  max_rows bounds the rows
 * (normally T), max_slots the slot tables, E the expert count of W1/W2 (slots naming an
 * expert outside [0,E) are skipped).  Rows outside all slots are not written.
 * row_index (may be NULL): fused gather.  When given, row r of the permuted row space is read
 * from x_perm[row_index[r]] -- pass the token matrix x as x_perm and moe_dispatch's perm as
 * row_index, and call moe_dispatch with x = x_perm = NULL: the permuted copy of the tokens is
 * then never written to HBM.  x_perm must hold max_rows rows; an index outside [0, max_rows)
 * is never dereferenced (the row is computed from a zero row or from row 0, its output is
 * unspecified).  y_perm stays in permuted row order either way.
 * Workspace layout: h occupies the first max_rows*F elements (row-major [max_rows, F], dtype) and
 * still holds the first product's output when the call's kernels have finished (rows outside all
 * slots are not written); the work lists follow it.
 */
size_t moe_expert_ffn_workspace_bytes(int max_rows, int max_slots, int d, int F, int dtype);
int moe_expert_ffn(const void *x_perm, const int32_t *row_index, const void *w1, const void *w2,
                   int weight_layout,
                   const int32_t *slot_offset, const int32_t *slot_expert, const int32_t *n_slots,
                   int max_rows, int max_slots, int E, int d, int F, int dtype, int schedule,
                   void *y_perm, void *ws, size_t ws_bytes, void *stream);

/* ---------------------------------------------------------------------------------------
 * moe_combine -- expert output scaled by the gate probability, back in token order; tokens
 * over capacity pass through unchanged (the replicated model keeps the baseline layer's
 * computation: Preliminaries, Conclusion).
 *   inv[s] >= 0 : out[s] = (residual ? x[s] : 0) + expert_prob[s] * y_perm[inv[s]]
 *                 (binary32 multiply-add, rounded once to dtype)
 *   inv[s] <  0 : out[s] = x[s]  bit for bit
 * out must not alias x or y_perm.  d*sizeof(element) a multiple of 16.
 */
int moe_combine(const void *y_perm, const void *x, const int32_t *inv, const float *expert_prob,
                int T, int d, int dtype, int residual, void *out, void *stream);

/* =======================================================================================
 * Measurement (not part of the method; used by the benchmark only).
 * moe_expert_ffn_timed: moe_expert_ffn_rows (with row_index NULL: moe_expert_ffn, n_x_rows =
 * max_rows) that also records three hipEvent_t handles (passed as void*, any may be NULL) on the
 * call's stream: before its first product's kernel, between the two products, after the second.
 * It keeps no state: the events belong to this one call.  Same outputs as the untimed calls.
 */
int moe_expert_ffn_timed(const void *x, int n_x_rows, const int32_t *row_index, const void *w1,
                         const void *w2, int weight_layout, const int32_t *slot_offset,
                         const int32_t *slot_expert, const int32_t *n_slots, int max_rows, int max_slots,
                         int E, int d, int F, int dtype, int schedule, void *y_perm, void *ws,
                         size_t ws_bytes, void *stream, void *ev_before, void *ev_between, void *ev_after);


/* Ceilings of this machine for kernels shaped like the library's own (the benchmark quotes roofline
 * fractions against them beside the nominal peaks).
 * moe_measure_stream_read: one launch that reads `bytes` (a multiple of 16) of device memory once, a
 *   contiguous region per workgroup, with plain (nontemporal = 0) or non-temporal 16-byte loads, from
 *   n_workgroups workgroups of 256 threads (0: eight per compute unit, 16 KB in flight each: the whole chip;
 *   1 .. number of compute units: one workgroup per unit, 128 KB in flight each: what that many units can
 *   pull from memory -- the rate that bounds a kernel which gives every expert slot to one workgroup).
 * moe_measure_mfma_bf16: one launch of `iters` iterations of 32 v_mfma_f32_32x32x16_bf16 per wavefront (one
 *   workgroup of 4 wavefronts per compute unit, 4 x 4 accumulator blocks each, the 256 x 256 tile kernel's
 *   instruction mix) on operands that change every step, kept in registers (from_lds = 0) or re-read from
 *   LDS (from_lds = 1); moe_measure_mfma_bf16_flops gives the floating-point operations of such a launch.
 * sink: device scratch of moe_measure_sink_bytes() bytes (nothing meaningful is written).  The caller times
 * the launches (events on the stream).
 */
size_t moe_measure_sink_bytes(void);
int moe_measure_stream_read(const void *buf, size_t bytes, int nontemporal, int n_workgroups, void *sink,
                            void *stream);
size_t moe_measure_mfma_bf16_flops(int iters);
int moe_measure_mfma_bf16(int iters, int from_lds, void *sink, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* MOE_MPMC_H */
