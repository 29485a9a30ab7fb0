/*
 * ape.h -- C ABI of the MI355X (gfx950) APE attention library.
 *
 * APE = Adaptive Parallel Encoding (arXiv 2502.05431).  The library computes
 * the attention of that method for ONE transformer layer:
 *
 *   ape_encode_chunks      offline pre-caching of N contexts (Section 2.2) that
 *                          share one prefix (Section 4.1): block-diagonal causal
 *                          attention, every context at the same positions.
 *   ape_attention_prefill  query rows over prefix + all cached contexts + the
 *   ape_attention_decode   query's own causal KV with the refined attention of
 *                          Section 4.4 ("Eq.5"): context scores use 1/(T sqrt d),
 *                          the pooled context partition sum is raised to S.
 *   ape_rope_write_cache   rotary embedding with positions re-used across contexts
 *                          (Section 1) fused with the KV-cache write, in front of the above.
 *   ape_attention_tree     the same over a tree of contexts with a scaling factor per
 *                          node (Appendix C.2 and C.5); S per context is one such tree.
 *
 * General conventions
 *   - Every data pointer marked DEVICE points to GPU memory owned by the caller;
 *     the library never allocates, frees or copies device memory and keeps no
 *     state between calls.  Pointers marked HOST are read during the call only.
 *     (The library depends on the HIP runtime alone.  Whole transformer layers around the
 *     attention, which need a GEMM library and its handle, are a separate shared object with a
 *     header of its own, ape_layer.h.)
 *   - Every data pointer is 16-byte aligned (rows of head_dim elements then are too: the kernels
 *     use 16-byte accesses); that holds for the pointers inside device tables (k_chunks[i], the
 *     caches of ape_rope_write_cache) as well, which the host cannot check.  Tables themselves are
 *     aligned to their element size.
 *   - Tensors are row-major [tokens, heads, head_dim]; K/V have n_kv_heads heads,
 *     Q/O have n_q_heads heads; query head h reads KV head h / (n_q_heads/n_kv_heads).
 *     Q and K arrive already position-rotated.
 *   - dtype APE_F32: fp32 in/out, fp32 arithmetic.  APE_BF16: bf16 in/out, bf16
 *     matrix-core products with fp32 accumulation and fp32 softmax.
 *   - Kernels are enqueued on `stream` (a hipStream_t passed as void*, NULL = the
 *     null stream); calls return without synchronising.
 *   - Return value: APE_OK or a negative ape_status.  Argument errors are found on
 *     the host before anything is launched and leave all outputs untouched.
 *     ape_last_error() gives a thread-local description of the last failure.
 *   - LogSumExp outputs are natural-log, fp32.
 *   - Size limits of one call (APE_ERR_UNSUPPORTED beyond, nothing launched): query calls write
 *     fewer than 2^24 (row, head) outputs (batch x q_len x n_q_heads); the attention launch of a tree
 *     call (split slots x KV heads x query tiles) has fewer than 2^24 workgroups; an encode on the matrix-core path
 *     launches contexts x n_kv_heads x ceil(longest context x heads-per-KV-head / 128) workgroups and
 *     takes fewer than 2^24 of them, on the other paths fewer than 2^26 (row, head) outputs.  Token
 *     counts are 32-bit (a call covers fewer than 2^31 tokens); byte offsets are 64-bit throughout.
 */
#ifndef APE_H
#define APE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    APE_OK = 0,
    APE_ERR_INVALID_ARG = -1,   /* null pointer, bad length, T or S not finite and > 0, ...      */
    APE_ERR_UNSUPPORTED = -2,   /* head_dim / head ratio / dtype the kernels do not cover, or a   */
                                /* call beyond the size limits above                              */
    APE_ERR_WORKSPACE = -3,     /* workspace missing or smaller than ape_workspace_bytes says     */
    APE_ERR_DEVICE = -4         /* HIP reported a launch error                                    */
} ape_status;

typedef enum { APE_F32 = 0, APE_BF16 = 1 } ape_dtype;
/* OR-ed into ape_shape.dtype: run the portable vector-ALU kernels even where the matrix-core
 * kernels apply.  Same results within tolerance; meant for cross-checking, not for speed. */
#define APE_DTYPE_FLAG_GENERIC 0x100
typedef enum { APE_OP_ENCODE = 0, APE_OP_PREFILL = 1, APE_OP_DECODE = 2 } ape_op;

/* Attention head geometry.  Supported: head_dim multiple of 8 and <= 256 for APE_F32 and
 * APE_BF16; n_q_heads a multiple of n_kv_heads.  bf16 with head_dim == 128 and
 * n_q_heads/n_kv_heads in {1,2,4,8} runs on the matrix-core kernels. */
typedef struct {
    int32_t n_q_heads;
    int32_t n_kv_heads;
    int32_t head_dim;
    int32_t dtype;              /* ape_dtype */
} ape_shape;

/*
 * One request's cached KV as the query sees it (Section 2.2 "Generating Response",
 * Section 4.4).  The contexts are used in place through a table, so that any subset
 * of pre-cached contexts can be attended without copying.
 */
typedef struct {
    const void *k_prefix;              /* DEVICE [prefix_len, n_kv_heads, head_dim]; may be NULL if prefix_len == 0 */
    const void *v_prefix;              /* DEVICE, same shape                                                         */
    int32_t prefix_len;                /* >= 0                                                                       */
    int32_t n_chunks;                  /* >= 0; 0 = no context (plain causal attention over prefix + self)          */
    const void *const *k_chunks;       /* DEVICE array [n_chunks] of DEVICE pointers, chunk i: [l_i, n_kv_heads, d] */
    const void *const *v_chunks;       /* DEVICE array [n_chunks] of DEVICE pointers                                */
    const int32_t *cu_chunk_lens;      /* DEVICE [n_chunks + 1]: 0, l_1, l_1+l_2, ..., total_ctx_len                */
    int32_t total_ctx_len;             /* HOST copy of cu_chunk_lens[n_chunks]; the caller keeps the two equal.     */
                                       /* Token counts are 32-bit: one request holds fewer than 2^31 context tokens */
                                       /* (4 TB of K at the Llama-3-8B shape, beyond any one GPU's memory)          */
    int32_t self_len;                  /* tokens in k_self/v_self INCLUDING the rows being queried; >= q_len >= 1   */
    const void *k_self;                /* DEVICE [self_len, n_kv_heads, head_dim]: query + generated tokens         */
    const void *v_self;                /* DEVICE                                                                     */
    float temperature;                 /* T of Eq.5, finite and > 0 (the paper uses T <= 1)                         */
    float scale;                       /* S of Eq.5, finite and > 0 (the paper uses S <= 1)                         */
} ape_request;

/*
 * Bytes of caller-provided DEVICE workspace an operation needs (0 is possible).
 * An upper bound that depends only on the arguments given, never on the data.
 *   op            ape_op
 *   batch         requests (decode, batched prefill); 1 for ape_attention_prefill; ignored for encode
 *   q_len         query rows per request (prefill); 1 for decode; ignored for encode
 *   max_total_kv  the largest total_ctx_len of any request the workspace will serve; the result
 *                 covers every call whose contexts are no longer than that.  Negative: no limit known,
 *                 the result then covers every context length (the most splits the planner ever uses).
 * Returns 0 on invalid arguments as well; the entry points re-validate.
 */
size_t ape_workspace_bytes(int op, const ape_shape *shape, int32_t batch, int32_t q_len, int64_t max_total_kv);

/*
 * Pre-caching attention of Section 2.2 with the shared prefix of Section 4.1.
 * Context i is encoded as [prefix ; C_i]: row r of context i attends to every prefix
 * token and to rows 0..r of its own context with scores q.k/sqrt(d) (Section 2.3);
 * contexts never see each other; no T, no S.
 *
 *   q_prefix/o_prefix   DEVICE [prefix_len, n_q_heads, d] or both NULL: when given, the
 *                       prefix rows are computed too (plain causal attention over the prefix).
 *   k_prefix,v_prefix   DEVICE [prefix_len, n_kv_heads, d]
 *   q_chunks,o_chunks   DEVICE packed contexts [M, n_q_heads, d], M = cu_chunk_lens_host[n_chunks]
 *   k_chunks,v_chunks   DEVICE packed contexts [M, n_kv_heads, d]
 *   cu_chunk_lens_host  HOST  [n_chunks + 1] prefix sums of the context lengths (sizes the grid)
 *   cu_chunk_lens_dev   DEVICE copy of the same array (read by the kernels)
 *   lse_prefix          DEVICE fp32 [n_q_heads, prefix_len] or NULL
 *   lse_chunks          DEVICE fp32 [n_q_heads, M] or NULL: LogSumExp of each row's scores
 *   workspace           unused by the current kernels (ape_workspace_bytes gives 0); may be NULL
 */
int ape_encode_chunks(const ape_shape *shape,
                      const void *q_prefix, const void *k_prefix, const void *v_prefix, int32_t prefix_len,
                      const void *q_chunks, const void *k_chunks, const void *v_chunks,
                      const int32_t *cu_chunk_lens_host, const int32_t *cu_chunk_lens_dev, int32_t n_chunks,
                      void *o_prefix, void *o_chunks, float *lse_prefix, float *lse_chunks,
                      void *workspace, size_t workspace_bytes, void *stream);

/*
 * Query prefill with the refined attention of Section 4.4 (Eq.5), computed in the
 * two-block form of Appendix C.3/C.4: context block with scores q.k/(T sqrt d) and its
 * LogSumExp multiplied by S, non-context block (prefix + causal self) unscaled, merged by
 * a softmax over the two LogSumExps.  S is applied to the POOLED context block.
 *
 *   req       HOST  one request; the last q_len tokens of k_self/v_self are the query rows'
 *             own KV: row r sees self tokens 0 .. self_len - q_len + r.
 *   q, out    DEVICE [q_len, n_q_heads, d]
 *   lse_out   DEVICE fp32 [n_q_heads, q_len] or NULL: log(Z_prefix + Z_ctx^S + Z_self)
 *   workspace DEVICE, >= ape_workspace_bytes(APE_OP_PREFILL, shape, 1, q_len, req->total_ctx_len), 256-byte aligned
 */
int ape_attention_prefill(const ape_shape *shape, const ape_request *req,
                          const void *q, int32_t q_len, void *out, float *lse_out,
                          void *workspace, size_t workspace_bytes, void *stream);

/*
 * Query prefill of a batch of independent requests with the same number of query rows (the
 * serving setting of Section 5.4 runs several queries at once): ape_attention_prefill for every
 * request, in one launch.  Each request has its own prefix, contexts, self KV, T and S.
 *
 *   reqs      HOST array [batch]
 *   q, out    DEVICE [batch, q_len, n_q_heads, d]
 *   lse_out   DEVICE fp32 [batch, n_q_heads, q_len] or NULL
 *   workspace DEVICE, >= ape_workspace_bytes(APE_OP_PREFILL, shape, batch, q_len, longest context), 256-byte aligned
 */
int ape_attention_prefill_batch(const ape_shape *shape, const ape_request *reqs, int32_t batch,
                                const void *q, int32_t q_len, void *out, float *lse_out,
                                void *workspace, size_t workspace_bytes, void *stream);

/*
 * One decode step for a batch of independent requests: Eq.5 with a single query row per
 * request, which sees all self_len self tokens (the newest being its own; the caller has
 * appended its K/V before the call).  Each request carries its own T and S.
 *
 *   reqs      HOST array [batch]
 *   q, out    DEVICE [batch, n_q_heads, d]
 *   lse_out   DEVICE fp32 [batch, n_q_heads] or NULL
 *   workspace DEVICE, >= ape_workspace_bytes(APE_OP_DECODE, shape, batch, 1, longest context), 256-byte aligned
 */
int ape_attention_decode(const ape_shape *shape, const ape_request *reqs, int32_t batch,
                         const void *q, void *out, float *lse_out,
                         void *workspace, size_t workspace_bytes, void *stream);

/*
 * ape_attention_decode for callers that cannot allocate device memory or pass a workspace (code
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc): the same decode
 * step, same kernels and same results, with the partial results of the context splits kept in a
 * fixed buffer of APE_STATIC_SCRATCH_BYTES that the library holds in the memory of every GPU it is
 * loaded on, until the process ends.  The call allocates and frees nothing.
 *
 *   reqs, batch, q, out, lse_out, stream   as for ape_attention_decode
 * A call whose partial results do not fit (about batch x n_q_heads x (splits + 1) x (head_dim + 1) x
 * 4 bytes; the Llama-3-8B shape fits 32 requests of 16K context tokens or one of 128K several times
 * over) returns APE_ERR_UNSUPPORTED with nothing launched.  All calls on one GPU share the one
 * buffer, which keeps the last call's contents: calls that overlap in time on the same GPU (two
 * streams, two host threads) race and must be serialised by the caller.  Nothing in it needs
 * clearing between calls.  The first call on a device looks the buffer's address up once (do it
 * outside a graph capture); the current device must be the stream's.
 */
#define APE_STATIC_SCRATCH_BYTES (8u << 20)
int ape_attention_decode_static(const ape_shape *shape, const ape_request *reqs, int32_t batch,
                                const void *q, void *out, float *lse_out, void *stream);

/*
 * One node of a tree of contexts (Appendix C.5: a cache whose contexts form a hierarchy).
 * Appendix C.2 is applied at every node: a node merges its children by a softmax over their
 * LogSumExp values A, and its own value is A_n = scale * LogSumExp(A_children).  The children
 * of a node are EITHER cached contexts (leaf_children != 0: contexts first .. first+count-1 of
 * the request's chunk table, each with the unscaled LogSumExp of its scores q.k/(T sqrt d))
 * OR nodes (leaf_children == 0: nodes first .. first+count-1).
 * Numbering: node 0 is the root; node children are numbered breadth-first, i.e. in the order
 * of their parents (the first non-leaf node's children start at 1, the next one's follow
 * directly, ...), so that every child index is above its parent's and every level of the tree
 * is one index range.  Every context of the chunk table belongs to exactly one node.
 */
typedef struct {
    float scale;                /* S_n, finite and > 0                                           */
    int32_t first;              /* first child: context index or node index                      */
    int32_t count;              /* number of children, >= 1                                      */
    int32_t leaf_children;      /* != 0: the children are contexts; 0: they are nodes            */
} ape_tree_node;

#define APE_TREE_MAX_NODES 2048
#define APE_TREE_MAX_CONTEXTS 4096
#define APE_TREE_MAX_DEPTH 16

/*
 * Bytes of DEVICE workspace ape_attention_tree needs for a request with total_ctx_len context
 * tokens, a tree of n_nodes nodes and q_len query rows (depends on these sizes only).
 * Returns 0 on invalid arguments.
 */
size_t ape_tree_workspace_bytes(const ape_shape *shape, int32_t total_ctx_len, int32_t n_nodes, int32_t q_len);

/*
 * Attention of q_len query rows of ONE request over prefix + a tree of cached contexts + own
 * causal KV: Appendix C.2 applied per node (Appendix C.5).  The result is
 * Softmax(A_other, A_root) [V_other, V_root] with "other" the unscaled block of prefix and
 * causal self tokens.  Two trees reproduce the flat forms: one node of scale S over all
 * contexts is ape_attention_prefill (pooled S, Eq.5); a root of scale 1 over one node of
 * scale S per context is Appendix C.2 as written (S per context).
 * The contexts of one node merge exactly (Appendix C.1) and are attended as one run of tokens;
 * partial results never mix contexts of different nodes, which is what the per-node scaling needs.
 *
 *   req            HOST  as for ape_attention_prefill; req->scale is not used (the nodes carry
 *                  the scaling factors) but must still be valid; n_chunks >= 1
 *   nodes_host     HOST  [n_nodes], validated before anything is launched
 *   nodes_dev      DEVICE copy of the same array (read by the kernels); the caller keeps the
 *                  two equal
 *   q, out         DEVICE [q_len, n_q_heads, d]; q_len == 1 is a decode step
 *   lse_out        DEVICE fp32 [n_q_heads, q_len] or NULL: log(exp(A_other) + exp(A_root))
 *   workspace      DEVICE, >= ape_tree_workspace_bytes(shape, req->total_ctx_len, n_nodes, q_len),
 *                  256-byte aligned
 * Limits: n_nodes <= APE_TREE_MAX_NODES, n_chunks <= APE_TREE_MAX_CONTEXTS, depth <=
 * APE_TREE_MAX_DEPTH levels of nodes (APE_ERR_UNSUPPORTED beyond).
 */
int ape_attention_tree(const ape_shape *shape, const ape_request *req,
                       const ape_tree_node *nodes_host, const ape_tree_node *nodes_dev, int32_t n_nodes,
                       const void *q, int32_t q_len, void *out, float *lse_out,
                       void *workspace, size_t workspace_bytes, void *stream);

/*
 * Rotary position embedding with positions re-used across contexts (Section 1, "Re-using
 * Positions": every context occupies the same range of positions), fused with the write of the
 * KV cache -- the step in front of ape_encode_chunks and of the query-time calls.
 * The packed rows [M, heads, d] are n_chunks segments given by cu_chunk_lens; token j of EVERY
 * segment has position position_offset + j.  Rotation: the published rotary embedding in
 * half-split pairing, dims (c, c + d/2) turn by pos * rope_base^(-2c/d); fp32 arithmetic on
 * angles reduced in fp64.  (Prefix: one segment at offset 0.  Contexts: offset prefix_len.
 * Query and generated tokens: one segment at offset prefix_len + max_i l_i.)
 *
 *   q_raw, q_rot   DEVICE packed [M, n_q_heads, d], or both NULL; q_rot may be q_raw (in place)
 *   k_raw          DEVICE packed [M, n_kv_heads, d] or NULL: rotated keys of segment i go to
 *   k_cache        DEVICE array [n_chunks] of DEVICE pointers, k_cache[i]: [l_i, n_kv_heads, d]
 *                  (views into one packed buffer are fine: that buffer then feeds ape_encode_chunks)
 *   v_raw, v_cache same for the values, which are copied unchanged; or both NULL
 *   cu_chunk_lens_host / _dev  HOST and DEVICE [n_chunks + 1] prefix sums of the segment lengths
 * head_dim must be even (it is a multiple of 8).  No workspace.
 */
int ape_rope_write_cache(const ape_shape *shape,
                         const void *q_raw, const void *k_raw, const void *v_raw,
                         const int32_t *cu_chunk_lens_host, const int32_t *cu_chunk_lens_dev, int32_t n_chunks,
                         int32_t position_offset, float rope_base,
                         void *q_rot, void *const *k_cache, void *const *v_cache, void *stream);

/* Text for a status code (static storage). */
const char *ape_status_string(int status);
/* Description of the calling thread's last failing call ("" if none). */
const char *ape_last_error(void);
/* Library version, "major.minor.patch". */
const char *ape_version(void);

#ifdef __cplusplus
}
#endif
#endif /* APE_H */
