/*
 * ape_layer.h -- C ABI of libape_layer.so: whole transformer layers around the encode attention of
 * the APE attention library (ape.h), for a per-layer / per-model latency of the context
 * pre-caching pass (arXiv 2502.05431, Section 2.2; Section 5.4 measures that pass end to end).
 *
 * A separate shared object on purpose: the four matrix products of a layer are rocBLAS GEMMs, so
 * this library links rocBLAS and keeps one rocBLAS handle per device (created at the first call on
 * that device, which allocates; bound to each call's stream).  The attention library itself stays
 * free of both.  Calls of this library are serialised by a process-wide lock while they enqueue
 * (two host threads may call at once; their launches do not interleave).  Under a HIP graph
 * capture the handle must already exist: make one plain call on the device first.
 * Conventions otherwise as in ape.h (DEVICE / HOST pointers, 16-byte alignment, status codes,
 * ape_last_error()).
 */
#ifndef APE_LAYER_H
#define APE_LAYER_H

#include "ape.h"

#ifdef __cplusplus
extern "C" {
#endif

/*
 * Weights of one transformer layer (the published Llama layer of the models the paper evaluates;
 * Section 5.4 measures their prefill).  All DEVICE, dtype of the shape, [out_features, in_features]
 * row-major.
 */
typedef struct {
    int32_t hidden;             /* model width, multiple of 8                                        */
    int32_t intermediate;       /* MLP width, multiple of 8                                          */
    float rms_eps;              /* RMSNorm epsilon                                                   */
    float rope_base;            /* rotary base                                                       */
    const void *attn_norm;      /* [hidden]                                                          */
    const void *w_qkv;          /* [(n_q_heads + 2 n_kv_heads) d, hidden]: Q rows, then K, then V    */
    const void *w_o;            /* [hidden, n_q_heads d]                                             */
    const void *mlp_norm;       /* [hidden]                                                          */
    const void *w_gate_up;      /* [2 intermediate, hidden]: gate rows, then up rows                 */
    const void *w_down;         /* [hidden, intermediate]                                            */
} ape_layer_weights;

/*
 * Optional DEVICE buffers that receive two intermediates of ape_layer_encode, so that the attention
 * inside the layer can be checked on its own inputs (either may be NULL):
 *   q_rot  [M, n_q_heads, d]   the rotated queries the attention reads
 *   attn   [M, n_q_heads, d]   the attention output, before the output projection
 * (the rotated keys and the values are the k_cache / v_cache outputs).
 */
typedef struct {
    void *q_rot;
    void *attn;
} ape_layer_taps;

/* Bytes of DEVICE workspace ape_layer_encode needs for total_rows packed context tokens. */
size_t ape_layer_workspace_bytes(const ape_shape *shape, int32_t hidden, int32_t intermediate, int32_t total_rows);
/* The same for ape_layers_encode over n_layers layers. */
size_t ape_layers_workspace_bytes(const ape_shape *shape, int32_t hidden, int32_t intermediate, int32_t total_rows,
                                  int32_t n_layers);

/*
 * One layer of the context pre-caching pass (Section 2.2) over the packed contexts:
 *   h = RMSNorm(x);  q, k, v = h Wqkv^T;  q, k rotated with positions re-used across contexts
 *   (Section 1: token j of every context at prefix_len + j);  k, v written to the cache;
 *   a = the attention of ape_encode_chunks (prefix KV + own context, causal);  x1 = x + a Wo^T;
 *   y = x1 + (SiLU(g) * u) Wd^T with [g, u] = RMSNorm(x1) Wgate_up^T.
 * The four matrix products are rocBLAS GEMMs with fp32 accumulation; everything between them runs
 * in this library's and the attention library's kernels.  Intermediate tensors have the dtype of
 * the shape.
 *
 *   x, y               DEVICE packed [M, hidden], M = cu_chunk_lens_host[n_chunks]; y may not alias x
 *   k_prefix, v_prefix DEVICE [prefix_len, n_kv_heads, d]: THIS layer's cached prefix KV (rotated)
 *   k_cache, v_cache   DEVICE packed [M, n_kv_heads, d]: receive this layer's context KV
 *   taps               HOST, or NULL
 *   workspace          DEVICE, >= ape_layer_workspace_bytes(shape, hidden, intermediate, M), 256-byte aligned
 */
int ape_layer_encode(const ape_shape *shape, const ape_layer_weights *weights, const void *x,
                     const void *k_prefix, const void *v_prefix, int32_t prefix_len,
                     const int32_t *cu_chunk_lens_host, const int32_t *cu_chunk_lens_dev, int32_t n_chunks,
                     void *k_cache, void *v_cache, void *y, const ape_layer_taps *taps,
                     void *workspace, size_t workspace_bytes, void *stream);

/*
 * A stack of n_layers such layers (the whole pre-caching pass of a model, embedding and final norm
 * aside): layer l reads the hidden states layer l-1 wrote, writes its own context KV to k_cache[l] /
 * v_cache[l] and attends over its own prefix KV k_prefix[l] / v_prefix[l].
 *
 *   layers               HOST  [n_layers]; all of the same hidden and intermediate width
 *   x, y                 DEVICE packed [M, hidden]: input of layer 0, output of the last layer
 *   k_prefix, v_prefix   HOST arrays [n_layers] of DEVICE pointers [prefix_len, n_kv_heads, d]
 *                        (may be NULL when prefix_len == 0)
 *   k_cache, v_cache     HOST arrays [n_layers] of DEVICE pointers, packed [M, n_kv_heads, d]
 *   workspace            DEVICE, >= ape_layers_workspace_bytes(shape, hidden, intermediate, M, n_layers)
 */
int ape_layers_encode(const ape_shape *shape, const ape_layer_weights *layers, int32_t n_layers, const void *x,
                      const void *const *k_prefix, const void *const *v_prefix, int32_t prefix_len,
                      const int32_t *cu_chunk_lens_host, const int32_t *cu_chunk_lens_dev, int32_t n_chunks,
                      void *const *k_cache, void *const *v_cache, void *y,
                      void *workspace, size_t workspace_bytes, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* APE_LAYER_H */
