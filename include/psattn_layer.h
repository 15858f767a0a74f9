/*
 * psattn_layer — a whole self-attention layer on prefix-shared sequences (C ABI,
 * libpsattn_layer.so; needs libpsattn.so and rocBLAS).
 *
 * x -> Q, K, V projections -> rotary embedding with the position ids of the paired format
 * (Section 3.1) -> prefix-shared attention -> output projection, forward and backward.
 * This is the "attention layer" micro-benchmark of the paper's Section 4.2, where the
 * projections (linear in the number of tokens) and the attention (quadratic) are timed
 * together on the prefix-shared and on the paired format.  The projections are plain
 * dense GEMMs (rocBLAS, bf16 operands, fp32 accumulation); the rest is libpsattn.
 *
 * All tensors bfloat16, device memory, row-major: X, Y, dX, dY [T, hidden]; weights in the
 * [out_features, in_features] convention (y = x W^T): Wq [n_q_heads * 128, hidden], Wk, Wv
 * [n_kv_heads * 128, hidden], Wo [hidden, n_q_heads * 128]; their gradients likewise.
 * head_dim 128 only.  The caller owns everything, including the workspace (at least
 * psattn_layer_workspace_bytes(); it carries the activations from psattn_layer_fwd to
 * psattn_layer_bwd, so the same buffer must be passed to both, untouched in between).
 * Calls are asynchronous on hip_stream.  Status codes as in psattn.h.
 */
#ifndef PSATTN_LAYER_H
#define PSATTN_LAYER_H

#include "psattn.h"

#ifdef __cplusplus
extern "C" {
#endif

typedef struct psattn_layer psattn_layer; /* opaque: shapes + a rocBLAS handle */

int psattn_layer_create(int32_t hidden, int32_t n_q_heads, int32_t n_kv_heads, int32_t head_dim, psattn_layer** out);
int psattn_layer_free(psattn_layer* layer);
size_t psattn_layer_workspace_bytes(const psattn_layer* layer, const psattn_meta* meta, int32_t total_tokens);

int psattn_layer_fwd(psattn_layer* layer, const psattn_meta* meta, const psattn_rope* rope, int32_t total_tokens,
                     float scale, const void* X, const void* Wq, const void* Wk, const void* Wv, const void* Wo,
                     void* Y, void* workspace, size_t workspace_bytes, void* hip_stream);

/* dX, dWq, dWk, dWv, dWo are fully overwritten (dX = dQ Wq + dK Wk + dV Wv is accumulated in
 * its bfloat16 storage across the three products). */
int psattn_layer_bwd(psattn_layer* layer, const psattn_meta* meta, const psattn_rope* rope, int32_t total_tokens,
                     float scale, const void* X, const void* Wq, const void* Wk, const void* Wv, const void* Wo,
                     const void* dY, void* dX, void* dWq, void* dWk, void* dWv, void* dWo,
                     void* workspace, size_t workspace_bytes, void* hip_stream);

#ifdef __cplusplus
}
#endif
#endif /* PSATTN_LAYER_H */
