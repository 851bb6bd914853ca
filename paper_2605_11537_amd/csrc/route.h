// Host-side launchers shared between source files.  route.hip's, which sru_predict reuses (its head is a router-shaped
// product + argmax, its projections need the same packed weight image).
#pragma once
#include "common.h"

namespace moe {
size_t route_ws_bytes(int d, int E, int dtype);
int route_launch(const void *x, const void *w_router, int w_layout, const float *b_router, int T, int d, int E,
                 int dtype, int top_k, int renormalize, int32_t *idx, float *prob, float *logits_opt, void *ws,
                 hipStream_t st, const char *who);
// in [K][N] bf16 row-major -> packed image (N a multiple of 32), 16-byte piece ((n/32)*(K/8) + k/8)*32 + n%32
int pack_matrix_launch(const void *in, int K, int N, void *out, hipStream_t st, const char *who);
// attention.hip: z = h + sparsemax-attention context over each of the B sequences of L states (bf16, n features)
size_t sru_attention_ws_bytes(int B, int L, int n);   // packed image of the states
int sru_attention_launch(const void *h, int B, int L, int n, void *z, void *ht_ws, hipStream_t st, const char *who);
// plan.hip: histograms of ids in blocks of plan_partial_block() ids, partial[b][E]
int plan_partial_block();
int plan_partial_launch(const int32_t *idx, int T, int E, int32_t *partial, hipStream_t st, const char *who);
// dispatch.hip: block histograms of the routed ids, then the permute kernel with the replica plan made inside
// it (from plan_partial, or from the routed ids' own counts when plan_partial is NULL)
size_t dispatch_block_hist_bytes(int T, int E);
int dispatch_planned_launch(const int32_t *expert_idx, int T, int n_tokens, int E, int slot_capacity, int budget,
                            int policy, const int32_t *plan_partial, int n_partial, int n_plan_ids,
                            int32_t *block_hist, int32_t *plan_counts, int32_t *replicas, int32_t *slot_base,
                            int32_t *slot_expert, int32_t *n_slots, int32_t *counts, int32_t *kept,
                            int32_t *expert_offset, int32_t *slot_offset, int32_t *perm, int32_t *inv,
                            int32_t *row_token, hipStream_t st, const char *who);
}  // namespace moe
