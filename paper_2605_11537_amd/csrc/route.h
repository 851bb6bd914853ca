// Host-side entry points of route.hip that sru_predict reuses (its head is a router-shaped
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
size_t sru_attention_ws_bytes(int B, int L, int n);   // transposed states
int sru_attention_launch(const void *h, int B, int L, int n, void *z, void *ht_ws, hipStream_t st, const char *who);
}  // namespace moe
